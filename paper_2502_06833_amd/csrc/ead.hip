// Host side of the Entropy Adaptive Decoding library: handle, weight re-tiling, the
// per-step scheduler (Algorithm 1's loop over a batch of independent sequences) and
// the C ABI declared in include/ead.h.  All arithmetic of the method runs in the
// kernels of linear.hpp / attention.hpp / entropy.hpp and the small kernels below.
#include "../../include/ead.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "attention.hpp"
#include "common.hpp"
#include "entropy.hpp"
#include "linear.hpp"
#include "state.hpp"
#include "fused.hpp"
#include "stream.hpp"

using namespace ead;

namespace {

thread_local std::string g_create_error;

// ======================================================================================
// small kernels: weight re-tiling, plan, embedding gather, LM-head finalisation
// ======================================================================================
enum PackMode { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATEUP = 2 };

// Row-major [N, K] sources -> tiled layout (see common.hpp).  One thread per 8 elements.
//  PACK_QKV     rows = [q; k; v]; inside every q/k head, packed rows (2i, 2i+1) are the
//               rotary pair (i, i + hd/2) so that a lane pair holds both halves.
//  PACK_GATEUP  packed rows (2i, 2i+1) = (gate row i, up row i).
template <typename WT>
__global__ __launch_bounds__(256) void k_pack_weights(const WT *s0, const WT *s1, const WT *s2, WT *dst,
                                                      int Np, int K, int mode, int hd, int NQ, int NK) {
    const int KC = K >> 5;
    const size_t chunk = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (chunk >= (size_t)Np * K / 8) return;
    const size_t tile = chunk >> 6;
    const int l = (int)(chunk & 63);
    const int rb = (int)(tile / KC), kc = (int)(tile % KC);
    const int p = rb * 16 + (l & 15), k = kc * 32 + (l >> 4) * 8;
    const WT *src;
    if (mode == PACK_PLAIN) src = s0 + (size_t)p * K;
    else if (mode == PACK_GATEUP) src = ((p & 1) ? s1 : s0) + (size_t)(p >> 1) * K;
    else {
        if (p < NQ + NK) {
            const int pp = p < NQ ? p : p - NQ;
            const int head = pp / hd, r = pp % hd, dim = (r >> 1) + (r & 1) * (hd >> 1);
            src = (p < NQ ? s0 : s1) + (size_t)(head * hd + dim) * K;
        } else src = s2 + (size_t)(p - NQ - NK) * K;
    }
    Vec8<WT> v; v.load(src + k);
    float f[8]; v.unpack(f);
    store8_w(dst + chunk * 8, f);            // bf16 weights are re-encoded as halves (exact, see common.hpp)
}

template <typename WT>
__global__ __launch_bounds__(256) void k_copy(const WT *src, WT *dst, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

constexpr int kAllowWords = 8;       // sequences a host-side allow mask can name (64 per word)

struct PlanArgs {
    SeqState s; Plan p;
    int batch, m, budget, limit_off, lm_mode, ignore_model, step;
    // When the two models' passes run side by side on two streams, the other stream may be changing
    // the state of ITS sequences while this plan is built.  The host names the sequences of this
    // pass (their state is at rest); all others are left out whatever their state reads.
    int use_allow; unsigned long long allow[kAllowWords];
};

// Rows of one forward pass of model m: for every sequence that m serves, the positions
// m has not consumed yet (one in steady decoding, more right after a switch).
// lm_mode 0: no logits; 1: last row of sequences whose chunk reaches the end; 2: every row.
__global__ __launch_bounds__(256) void k_plan(PlanArgs a) {
    extern __shared__ int sm[];
    int *s_off = sm, *s_n = sm + a.batch, *s_have = sm + 2 * a.batch;
    const int tid = threadIdx.x;
    if (tid == 0) {
        int off = 0, nlm = 0;
        for (int b = 0; b < a.batch; ++b) {
            const bool allowed = !a.use_allow || ((a.allow[b >> 6] >> (b & 63)) & 1ull);
            const bool active = allowed && !a.s.done[b] && (a.ignore_model || a.s.model[b] == a.m) &&
                                (a.step < 0 || a.s.last_step[b] != a.step) &&
                                (a.ignore_model || a.s.ngen[b] < a.s.goal[b]);
            const int target = a.s.len[b] - a.limit_off, have = a.s.kvlen[a.m * a.s.max_batch + b];
            int n = active ? max(0, target - have) : 0;
            n = min(n, a.budget - off);
            s_off[b] = off; s_n[b] = n; s_have[b] = have;
            if (a.lm_mode == 1 && n > 0 && have + n == target) { a.p.lm_row[nlm] = off + n - 1; a.p.lm_seq[nlm] = b; ++nlm; }
            off += n;
        }
        a.p.hdr[0] = off;
        a.p.hdr[1] = a.lm_mode == 2 ? off : nlm;
    }
    __syncthreads();
    for (int b = 0; b < a.batch; ++b) {
        const int off = s_off[b], n = s_n[b], have = s_have[b];
        for (int j = tid; j < n; j += 256) {
            a.p.row_seq[off + j] = b; a.p.row_pos[off + j] = have + j;
            if (a.lm_mode == 2) { a.p.lm_row[off + j] = off + j; a.p.lm_seq[off + j] = b; }
        }
    }
    for (int b = tid; b < a.batch; b += 256) a.s.kvlen[a.m * a.s.max_batch + b] = s_have[b] + s_n[b];
}

template <typename WT>
__global__ __launch_bounds__(256) void k_embed(const WT *embed, const int *tokens, const int *hdr, const int *row_seq,
                                               const int *row_pos, int max_seq, int d, float *x) {
    const int t = blockIdx.x;
    if (t >= hdr[0]) return;
    const int tok = tokens[(size_t)row_seq[t] * max_seq + row_pos[t]];
    const WT *src = embed + (size_t)tok * d;
    for (int k = threadIdx.x * 8; k < d; k += 2048) {
        Vec8<WT> v; v.load(src + k);
        float f[8]; v.unpack(f);
        store8<float>(x + (size_t)t * d + k, f);
    }
}

// entropy-only finalisation for ead_entropy_argmax
__global__ __launch_bounds__(64) void k_entropy_finalize(const EntPartial *partials, int n_part, int rows, int unit,
                                                         float *H, int *argmax) {
    const int r = blockIdx.x;
    if (r >= rows) return;
    const EntStat st = merge_partials(partials + (size_t)r * n_part, n_part);
    if (threadIdx.x == 0) { H[r] = entropy_from(st, unit); if (argmax) argmax[r] = st.idx; }
}

// ======================================================================================
// host structures
// ======================================================================================
struct Layer { void *wqkv, *wo, *wgu, *wdown; float *g_attn, *g_ffn; void *kcache, *vcache, *vtcache; };

struct Model {
    int L, d, H, KV, hd, F, V, dtype;
    float eps, theta;
    void *embed, *lm_head; float *g_final; float2 *rope;
    std::vector<Layer> layers;
    double weight_bytes_nolm, lm_bytes, kv_bytes_per_pos, n_params;
    void *fused_mats = nullptr, *fused_layers = nullptr; int n_mats = 0; bool fused_ok = false;
    void *arena = nullptr; size_t layer_elems = 0, mat_off[4] = {0, 0, 0, 0};      // packed layer matrices: layer l's j-th at arena + l * layer_elems + mat_off[j]
    bool stream_ok = false;                                                     // k_decode_stream serves this model
    size_t esz() const { return dtype == EAD_BF16 ? 2 : 4; }
};

struct HostSeq { int len, kvlen[2], model, c, ngen, done, last_step, goal; };

}  // namespace

// Everything one forward pass writes besides the per-sequence state and its model's KV cache.
// There are two sets, and the second has a stream of its own, so that a pass of the small model
// and a pass of the large model can run side by side (they serve disjoint sequences).
struct LaneSet {
    hipStream_t stream = nullptr;
    float *x = nullptr, *q = nullptr, *o = nullptr, *hbuf = nullptr;
    bf16_t *xp_a = nullptr, *xp_o = nullptr, *xp_h = nullptr;
    float *sk_part = nullptr; int *sk_tickets = nullptr;
    float *part_o = nullptr; float2 *part_ml = nullptr; int *tickets = nullptr; EntPartial *lm_part = nullptr;
    Plan plan{};
    int *rb_model = nullptr, *rb_done = nullptr;      // pinned: what the host reads back after a pass
    hipEvent_t done_ev = nullptr;
};

struct ead_handle {
    Model mdl[2];
    ead_params prm;
    hipStream_t stream;
    int Tmax, items_max, lm_grid, score_rows, n_cu = 256;
    size_t lds_per_block = 65536;        // most LDS one workgroup may ask for on this device
    SeqState s; Plan plan; GateCfg cfg;
    // scratch
    float *x, *q, *o, *hbuf; bf16_t *xp_a, *xp_o, *xp_h;
    float *sk_part; int *sk_tickets;     // split-K partial sums of the MFMA path
    float *part_o; float2 *part_ml; int *tickets; EntPartial *lm_part; float *logits_dump; float *sc_H; int *sc_arg;
    int *h_model, *h_done;   // pinned
    LaneSet lanes[2]; int cur_lane = 0, two_lanes = 0; hipStream_t lane1_stream = nullptr;
    // fused single-row decode
    float *att_o; float2 *att_ml; unsigned *bar_mem; int *abort_flag; unsigned bar_epoch = 0; int fused_on = 0, fused_grid = 0;
    std::vector<void *> allocs;
    std::vector<HostSeq> hs;
    int batch, max_new, began, replay, n_new, force_model, step;
    int prefilled = 0;                   // both caches hold the prompts of the last ead_begin and nothing has clobbered them
    std::vector<int> prompt_len;
    int sched_grouped = 0, sched_phase = 0; float sched_hi = 0.5f, sched_lo = 0.25f;
    unsigned char attn_order[kAttnOrderMax]; int attn_order_n = 0;      // run_pass -> forward_pass: rows by falling context
    float samp_temp = 0.f; uint64_t samp_seed = 0;        // temperature 0: greedy
    int scoring = 0;                                       // inside ead_score: logits of given tokens, nothing is sampled
    ead_stats stats;
    std::string err;
    // optional per-kernel event timing
    int prof_on = 0;
    unsigned long long prof_mask = ~0ull;    // kernel classes (kind * 2 + model) that are bracketed while prof_on
    struct ProfRec { int cls; hipEvent_t a, b; double bytes; };
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> ev_pool;
    double prof_ms[64] = {0}, prof_bytes[64] = {0};
    int64_t prof_n[64] = {0};
};

namespace {

ead_status fail(ead_handle *h, ead_status st, const char *fmt, ...) {
    char buf[512];
    va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
    if (h) h->err = buf; else g_create_error = buf;
    return st;
}

// the scratch set and stream the launches that follow use
void use_lane(ead_handle *h, int i) {
    if (!h->two_lanes) i = 0;
    const LaneSet &l = h->lanes[i];
    h->stream = l.stream;
    h->x = l.x; h->q = l.q; h->o = l.o; h->hbuf = l.hbuf;
    h->xp_a = l.xp_a; h->xp_o = l.xp_o; h->xp_h = l.xp_h;
    h->sk_part = l.sk_part; h->sk_tickets = l.sk_tickets;
    h->part_o = l.part_o; h->part_ml = l.part_ml; h->tickets = l.tickets; h->lm_part = l.lm_part;
    h->plan = l.plan;
    h->cur_lane = i;
}
void save_lane(ead_handle *h, int i) {
    LaneSet &l = h->lanes[i];
    l.x = h->x; l.q = h->q; l.o = h->o; l.hbuf = h->hbuf;
    l.xp_a = h->xp_a; l.xp_o = h->xp_o; l.xp_h = h->xp_h;
    l.sk_part = h->sk_part; l.sk_tickets = h->sk_tickets;
    l.part_o = h->part_o; l.part_ml = h->part_ml; l.tickets = h->tickets; l.lm_part = h->lm_part;
    l.plan = h->plan;
}

enum ProfKind { PK_EMBED = 0, PK_PACK_ACT, PK_FMA_QKV, PK_FMA_RES, PK_FMA_SWIGLU, PK_FMA_LOGITS, PK_MFMA_QKV,
                PK_MFMA_RES, PK_MFMA_SWIGLU, PK_MFMA_LOGITS, PK_ATTN, PK_PLAN, PK_FINALIZE,
                PK_FUSED, PK_COUNT };
const char *const kProfNames[PK_COUNT] = {"embed", "pack_act", "linear_fma_qkv", "linear_fma_res", "linear_fma_swiglu",
                                          "linear_fma_logits", "linear_mfma_qkv", "linear_mfma_res", "linear_mfma_swiglu",
                                          "linear_mfma_logits", "attention", "plan", "lm_finalize",
                                          "decode_fused"};

// Brackets the launches made during its lifetime with two events (profiling mode only).
struct ProfScope {
    ead_handle *h; bool on;
    ProfScope(ead_handle *h_, int kind, int model, double bytes)
        : h(h_), on(h_->prof_on != 0 && ((h_->prof_mask >> (kind * 2 + model)) & 1ull)) {
        if (!on) return;
        hipEvent_t ev[2];
        for (auto &e : ev) {
            if (!h->ev_pool.empty()) { e = h->ev_pool.back(); h->ev_pool.pop_back(); }
            else if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
        }
        (void)hipEventRecord(ev[0], h->stream);
        h->prof_recs.push_back({kind * 2 + model, ev[0], ev[1], bytes});
    }
    ~ProfScope() { if (on) (void)hipEventRecord(h->prof_recs.back().b, h->stream); }
};

void prof_collect(ead_handle *h) {
    for (auto &r : h->prof_recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) { h->prof_ms[r.cls] += ms; h->prof_bytes[r.cls] += r.bytes; h->prof_n[r.cls]++; }
        h->ev_pool.push_back(r.a); h->ev_pool.push_back(r.b);
    }
    h->prof_recs.clear();
}

#define HIP_TRY(h, expr)                                                                         \
    do { hipError_t e_ = (expr);                                                                 \
         if (e_ != hipSuccess)                                                                   \
             return fail(h, e_ == hipErrorOutOfMemory ? EAD_ERR_OOM : EAD_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

template <typename T>
ead_status dmalloc(ead_handle *h, T **p, size_t n) {
    void *v = nullptr;
    hipError_t e = hipMalloc(&v, std::max<size_t>(n * sizeof(T), 256));
    if (e != hipSuccess) return fail(h, EAD_ERR_OOM, "hipMalloc of %zu bytes failed: %s", n * sizeof(T), hipGetErrorString(e));
    h->allocs.push_back(v);
    *p = (T *)v;
    return EAD_OK;
}
#define TRY(expr) do { ead_status s_ = (expr); if (s_ != EAD_OK) return s_; } while (0)

ead_status check_model(const ead_model_desc *m, const char *name) {
    if (!m) return fail(nullptr, EAD_ERR_INVALID_ARG, "%s model is null", name);
    if (m->n_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->n_kv_heads < 1 || m->head_dim < 1 || m->d_ffn < 1 || m->vocab < 1)
        return fail(nullptr, EAD_ERR_INVALID_ARG, "%s model: non-positive dimension", name);
    if (m->dtype != EAD_F32 && m->dtype != EAD_BF16) return fail(nullptr, EAD_ERR_INVALID_ARG, "%s model: unknown dtype", name);
    if (m->d_model % 32 || m->d_ffn % 32 || m->vocab % 16 || (m->n_heads * m->head_dim) % 32)
        return fail(nullptr, EAD_ERR_SHAPE, "%s model: d_model, d_ffn, n_heads*head_dim must be multiples of 32 and vocab of 16", name);
    if (m->head_dim != 32 && m->head_dim != 64 && m->head_dim != 128)
        return fail(nullptr, EAD_ERR_SHAPE, "%s model: head_dim must be 32, 64 or 128", name);
    if (m->n_heads % m->n_kv_heads) return fail(nullptr, EAD_ERR_SHAPE, "%s model: n_heads not a multiple of n_kv_heads", name);
    const int G = m->n_heads / m->n_kv_heads;
    if (G < 1 || G > 8)
        return fail(nullptr, EAD_ERR_SHAPE, "%s model: n_heads/n_kv_heads must be between 1 and 8", name);
    if (m->dtype == EAD_F32 && (m->d_model > 4096 || m->d_ffn > 4096))
        return fail(nullptr, EAD_ERR_SHAPE, "%s model: float32 weights are supported up to width 4096", name);
    if (m->d_ffn > 15360 || m->d_model > 15360) return fail(nullptr, EAD_ERR_SHAPE, "%s model: width above 15360", name);
    if (!m->embed || !m->wq || !m->wk || !m->wv || !m->wo || !m->w_gate || !m->w_up || !m->w_down || !m->norm_attn ||
        !m->norm_ffn || !m->norm_final || !m->lm_head)
        return fail(nullptr, EAD_ERR_INVALID_ARG, "%s model: null weight pointer", name);
    for (int l = 0; l < m->n_layers; ++l)
        if (!m->wq[l] || !m->wk[l] || !m->wv[l] || !m->wo[l] || !m->w_gate[l] || !m->w_up[l] || !m->w_down[l] ||
            !m->norm_attn[l] || !m->norm_ffn[l])
            return fail(nullptr, EAD_ERR_INVALID_ARG, "%s model: null weight pointer in layer %d", name, l);
    return EAD_OK;
}

// `place`: where the packed matrix goes; null = memory of its own
template <typename WT>
ead_status pack_matrix(ead_handle *h, const void *s0, const void *s1, const void *s2, void **dst, int Np, int K,
                       int mode, int hd, int NQ, int NK, WT *place = nullptr) {
    WT *d = place;
    if (!d) TRY(dmalloc(h, &d, (size_t)Np * K));
    const size_t chunks = (size_t)Np * K / 8;
    hipLaunchKernelGGL(k_pack_weights<WT>, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, h->stream,
                       (const WT *)s0, (const WT *)s1, (const WT *)s2, d, Np, K, mode, hd, NQ, NK);
    *dst = d;
    return EAD_OK;
}

template <typename WT>
ead_status build_model(ead_handle *h, const ead_model_desc *src, Model *m, int max_batch, int max_seq) {
    m->L = src->n_layers; m->d = src->d_model; m->H = src->n_heads; m->KV = src->n_kv_heads; m->hd = src->head_dim;
    m->F = src->d_ffn; m->V = src->vocab; m->dtype = src->dtype; m->eps = src->rms_eps; m->theta = src->rope_theta;
    const int d = m->d, hd = m->hd, NQ = m->H * hd, NK = m->KV * hd;
    WT *e = nullptr;
    TRY(dmalloc(h, &e, (size_t)m->V * d));
    HIP_TRY(h, hipMemcpyAsync(e, src->embed, (size_t)m->V * d * sizeof(WT), hipMemcpyDeviceToDevice, h->stream));
    m->embed = e;
    TRY(pack_matrix<WT>(h, src->lm_head, nullptr, nullptr, &m->lm_head, m->V, d, PACK_PLAIN, 0, 0, 0));
    TRY(dmalloc(h, &m->g_final, (size_t)d));
    HIP_TRY(h, hipMemcpyAsync(m->g_final, src->norm_final, d * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
    m->layers.resize(m->L);
    const size_t cache_elems = (size_t)max_batch * m->KV * max_seq * hd;
    // The four matrices of all layers share one allocation with a constant layer stride, so that a
    // kernel that walks the whole model (k_decode_stream) finds every matrix by arithmetic alone.
    const size_t n_qkv = (size_t)(NQ + 2 * NK) * d, n_o = (size_t)d * NQ, n_gu = 2 * (size_t)m->F * d, n_dn = (size_t)d * m->F;
    const size_t layer_elems = n_qkv + n_o + n_gu + n_dn;        // every part a multiple of 512 elements
    WT *arena = nullptr;
    TRY(dmalloc(h, &arena, layer_elems * (size_t)m->L));
    m->arena = arena; m->layer_elems = layer_elems;
    m->mat_off[0] = 0; m->mat_off[1] = n_qkv; m->mat_off[2] = n_qkv + n_o; m->mat_off[3] = n_qkv + n_o + n_gu;
    for (int l = 0; l < m->L; ++l) {
        Layer &ly = m->layers[l];
        WT *lb = arena + (size_t)l * layer_elems;
        TRY(pack_matrix<WT>(h, src->wq[l], src->wk[l], src->wv[l], &ly.wqkv, NQ + 2 * NK, d, PACK_QKV, hd, NQ, NK, lb + m->mat_off[0]));
        TRY(pack_matrix<WT>(h, src->wo[l], nullptr, nullptr, &ly.wo, d, NQ, PACK_PLAIN, 0, 0, 0, lb + m->mat_off[1]));
        TRY(pack_matrix<WT>(h, src->w_gate[l], src->w_up[l], nullptr, &ly.wgu, 2 * m->F, d, PACK_GATEUP, 0, 0, 0, lb + m->mat_off[2]));
        TRY(pack_matrix<WT>(h, src->w_down[l], nullptr, nullptr, &ly.wdown, d, m->F, PACK_PLAIN, 0, 0, 0, lb + m->mat_off[3]));
        TRY(dmalloc(h, &ly.g_attn, (size_t)d)); TRY(dmalloc(h, &ly.g_ffn, (size_t)d));
        HIP_TRY(h, hipMemcpyAsync(ly.g_attn, src->norm_attn[l], d * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
        HIP_TRY(h, hipMemcpyAsync(ly.g_ffn, src->norm_ffn[l], d * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
        WT *kc = nullptr, *vc = nullptr;
        TRY(dmalloc(h, &kc, cache_elems)); TRY(dmalloc(h, &vc, cache_elems));
        ly.kcache = kc; ly.vcache = vc; ly.vtcache = nullptr;
        if (std::is_same<WT, bf16_t>::value && max_seq % 32 == 0) {
            // the matrix-core attention reads whole 32-key blocks of this copy and multiplies what lies
            // past a row's last key by zero: it must never hold anything but finite values
            WT *vt = nullptr;
            TRY(dmalloc(h, &vt, cache_elems));
            HIP_TRY(h, hipMemsetAsync(vt, 0, cache_elems * sizeof(WT), h->stream));
            ly.vtcache = vt;
        }
    }
    // rotary table in double precision: angle = pos * theta^(-2i/hd)
    std::vector<float2> tab((size_t)max_seq * (hd / 2));
    for (int i = 0; i < hd / 2; ++i) {
        const double inv = pow((double)m->theta, -2.0 * (double)i / (double)hd);
        for (int p = 0; p < max_seq; ++p) {
            const double ang = (double)p * inv;
            tab[(size_t)p * (hd / 2) + i] = make_float2((float)cos(ang), (float)sin(ang));
        }
    }
    TRY(dmalloc(h, &m->rope, tab.size()));
    HIP_TRY(h, hipMemcpyAsync(m->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));   // tab goes out of scope
    // tables for the fused single-row decode kernel
    {
        std::vector<FusedMat<WT>> mats;
        std::vector<FusedLayer<WT>> lys;
        for (int l = 0; l < m->L; ++l) {
            const Layer &ly = m->layers[l];
            mats.push_back({(const WT *)ly.wqkv, (NQ + 2 * NK) / 16, d / 32, 1});
            mats.push_back({(const WT *)ly.wo, d / 16, NQ / 32, 0});
            mats.push_back({(const WT *)ly.wgu, 2 * m->F / 16, d / 32, 0});
            mats.push_back({(const WT *)ly.wdown, d / 16, m->F / 32, 0});
            lys.push_back({ly.g_attn, ly.g_ffn, (WT *)ly.kcache, (WT *)ly.vcache, (WT *)ly.vtcache});
        }
        mats.push_back({(const WT *)m->lm_head, m->V / 16, d / 32, 0});
        m->n_mats = (int)mats.size();
        FusedMat<WT> *dm = nullptr; FusedLayer<WT> *dl = nullptr;
        TRY(dmalloc(h, &dm, mats.size())); TRY(dmalloc(h, &dl, lys.size()));
        HIP_TRY(h, hipMemcpy(dm, mats.data(), mats.size() * sizeof(mats[0]), hipMemcpyHostToDevice));
        HIP_TRY(h, hipMemcpy(dl, lys.data(), lys.size() * sizeof(lys[0]), hipMemcpyHostToDevice));
        m->fused_mats = dm; m->fused_layers = dl;
    }
    const double per_layer = (double)d * (NQ + 2 * NK) + (double)NQ * d + 3.0 * (double)d * m->F;
    m->n_params = m->L * (per_layer + 2.0 * d) + d + (double)m->V * d;
    m->weight_bytes_nolm = (m->L * per_layer) * sizeof(WT) + (2.0 * m->L + 1) * d * 4.0;
    m->lm_bytes = (double)m->V * d * sizeof(WT);
    m->kv_bytes_per_pos = 2.0 * m->L * NK * sizeof(WT);
    return EAD_OK;
}

// ======================================================================================
// one forward pass of one model over the rows of the current plan
// ======================================================================================
template <typename WT, int EPI>
void launch_valu(ead_handle *h, int mi, LinArgs<WT> &a, int T, int grid) {
    ProfScope ps(h, PK_FMA_QKV + EPI, mi, (double)a.Np * a.K * sizeof(WT));
    const int KC = a.K / 32;
    const size_t budget = 60 * 1024;
    int TC = 4;
    while (TC > 1 && ((size_t)TC * a.K * 4 + 8 * TC * 16 * 4 > budget || TC / 2 >= T)) TC >>= 1;
    const bool wide = std::is_same<WT, bf16_t>::value && KC >= 64;
    const int NW = wide ? 8 : 4;
    const size_t lds = (size_t)TC * a.K * 4 + (size_t)NW * TC * 16 * 4;
#define EAD_LV(TC_, NW_) hipLaunchKernelGGL((k_linear_valu<WT, TC_, NW_, EPI>), dim3(grid), dim3(NW_ * 64), lds, h->stream, a)
    if constexpr (std::is_same<WT, bf16_t>::value) {
        if (wide) { if (TC == 4) EAD_LV(4, 8); else if (TC == 2) EAD_LV(2, 8); else EAD_LV(1, 8); }
        else { if (TC == 4) EAD_LV(4, 4); else if (TC == 2) EAD_LV(2, 4); else EAD_LV(1, 4); }
    } else {
        if (TC == 4) EAD_LV(4, 4); else if (TC == 2) EAD_LV(2, 4); else EAD_LV(1, 4);
    }
#undef EAD_LV
}

// T: the host's count of token rows.  The shape of the matrix and ceil(T / 16) pick the kernel:
//  * large matrices, more than 32 rows (QKV and residual projections: more than 16): k_linear_mfma_ls, 64 to 128
//    rows per sweep, eight (gate/up: seven) row blocks per workgroup; where that gives fewer workgroups than
//    compute units, K is split over workgroups and k_sk_merge adds the slabs.  k_linear_mfma_wt is the
//    fallback should the device not grant the LDS k_linear_mfma_ls asks for;
//  * passes of 32 token blocks or more (prefill): no split of K; every matrix takes one workgroup per
//    (row-block group, sweep), the large ones in 128 x 256 tiles (k_linear_mfma_gemm) where those fill the chip;
//  * large matrices at fewer rows, and the LM head: k_linear_mfma with four waves
//    of four row blocks each (an activation tile is fetched once for four weight tiles) where
//    there are many row blocks, else with K split over KS workgroups per group of four row blocks
//    so that the chip still gets about two workgroups per compute unit (the last to arrive adds
//    the slabs), or eight waves that split K inside a workgroup of two row blocks (QKV);
//  * small matrices are latency-bound: one row block per four-wave workgroup, as many
//    workgroups as possible.
// NT token blocks per sweep follow T; the ring depth D follows the register budget.
constexpr float kSmallLaneMin = 0.3f;                  // grouped schedule, two lanes: see decode_grouped
constexpr int kSplitKGroups = 4096;                     // arrival counters
constexpr size_t kSplitKFloats = (size_t)8 << 20;      // partial sums: KS slabs of (padded Np) x 128 floats at most

// Kernels that ask for more than 64 KB of dynamic LDS have to say so once.
std::mutex g_lds_attr_mutex;
bool allow_big_lds(const void *kernel, size_t bytes) {
    static std::vector<const void *> done;
    std::lock_guard<std::mutex> lock(g_lds_attr_mutex);
    if (std::find(done.begin(), done.end(), kernel) != done.end()) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) { (void)hipGetLastError(); return false; }
    done.push_back(kernel);
    return true;
}

template <int EPI, bool SK, int NW, int RG>
bool launch_ls(ead_handle *h, const LinArgs<bf16_t> &a, int grid) {
    const void *kern = (const void *)k_linear_mfma_ls<EPI, SK, NW, RG>;
    const size_t lds = kLsLdsBytes(NW);
    if (lds > h->lds_per_block || !allow_big_lds(kern, lds)) return false;
    hipLaunchKernelGGL((k_linear_mfma_ls<EPI, SK, NW, RG>), dim3(grid), dim3((NW + kLsProducers) * 64), lds, h->stream, a);
    return true;
}

template <int EPI>
void launch_mfma(ead_handle *h, int mi, LinArgs<bf16_t> &a, int T, int grid_cap = 0) {
    ProfScope ps(h, PK_MFMA_QKV + EPI, mi, (double)a.Np * a.K * 2.0);
    const int NB = a.Np / 16, TB = (T + 15) / 16;
    const bool big = (double)a.Np * a.K * 2.0 >= 24e6;
    const int NT = TB <= 1 ? 1 : (TB == 2 ? 2 : 4);
    int cfg = !big ? 1 : (NB >= 4 * 256 ? 4 : 2);       // 1: (4 waves, R=1)  4: (4, R=4)  2: (8 waves, R=2)  5: (4, R=4, split K)
    // 3: (4 waves, R=2) for matrices below that size with many row blocks, from 33 rows up: with one row block per
    // workgroup every workgroup fetches all activation tiles for 16 output rows (gate/up of a narrow model:
    // 139 MB of activation reads beside 17 MB of weights)
    if constexpr (EPI == EPI_SWIGLU) { if (!big && NB >= 2 * h->n_cu && TB >= 3) cfg = 3; }
    const int rpw = cfg == 3 ? 2 : cfg;                  // row blocks per workgroup
    int grid = (NB + rpw - 1) / rpw;
    if constexpr (EPI != EPI_LOGITS) {
        // more than 32 rows: 64 to 128 rows per sweep, weight tiles shared through LDS.  Matrices with few
        // row blocks are split along K over workgroups; a second kernel adds the slabs in order and
        // runs the epilogue.  Passes of two or three sweeps (teacher-forced scoring) take one launch pair per
        // sweep, or one workgroup per (group, sweep) where K is not split; longer ones (prefill) see below.
        // (17-32 rows: measured better for the split-K matrices, 32 against 34 us, not for gate/up, 72 against 69)
        if ((big && (TB > 2 || (TB == 2 && EPI != EPI_SWIGLU))) || TB >= 4 * kWideTok) {
            // token blocks per sweep: four up to 64 rows; the pass's own five to eight for 65-128 rows, one
            // wave per block; eight for the sweeps of longer passes
            const bool multi = TB > kWideTok;
            const int NG = (NB + 7) / 8, nt = TB <= 4 ? 4 : (multi ? kWideTok : TB);
            // passes of four sweeps or more: one workgroup per (group, sweep) for every matrix.  Cost of a
            // launch in cycles per k tile: rounds of workgroups over the compute units times the time of a k
            // step (measured: about 260 + 64 rg cycles with rg row blocks x 128 rows, about 1150 for the
            // 128 x 256 tiles, which move twice the rows per step but are bound by what a compute unit
            // can fetch); the 128 x 256 tiles win where their groups still fill the chip
            const bool longpass = TB >= 4 * kWideTok;
            int rg_long = 8;
            if (longpass) {
                const int sw = (TB + kWideTok - 1) / kWideTok, n_cu = h->n_cu;
                auto cost_of = [&](int r) { return (((long)((NB + r - 1) / r) * sw + n_cu - 1) / n_cu) * (260 + 64 * r); };
                long cost = -1;
                if (EPI != EPI_QKV && cfg == 4) { rg_long = (NB + 6) / 7 <= n_cu ? 7 : 8; cost = cost_of(rg_long); }
                else for (int r = 8; r >= 5; --r) if (cost < 0 || cost_of(r) < cost) { cost = cost_of(r); rg_long = r; }
                const int sg = (TB + kGemmTok - 1) / kGemmTok;
                const long cost_gemm = (((long)NG * sg + n_cu - 1) / n_cu) * 1150;
                const void *kern = (const void *)k_linear_mfma_gemm<EPI>;
                if (big && cost_gemm < cost && kGemmLdsBytes <= h->lds_per_block && allow_big_lds(kern, kGemmLdsBytes)) {
                    a.sweeps = sg;
                    hipLaunchKernelGGL((k_linear_mfma_gemm<EPI>), dim3((NG + 7) / 8 * 8 * sg), dim3(640), kGemmLdsBytes, h->stream, a);
                    return;
                }
            }
            if constexpr (EPI != EPI_QKV) if (cfg == 4) {
                // seven row blocks per workgroup where that still fits one workgroup per compute unit
                // (1728 row blocks: 247 workgroups instead of 216 on 256 units)
                const int rg = (NB + 6) / 7 <= h->n_cu ? 7 : 8, ng = (NB + rg - 1) / rg;
                a.sweeps = (TB + nt - 1) / nt;
                const int grid_wt = a.sweeps > 1 ? (ng + 7) / 8 * 8 * a.sweeps : ng;
#define EAD_WT(TPW_, NW_) do { if (rg == 7) hipLaunchKernelGGL((k_linear_mfma_wt<6, EPI, false, TPW_, 7, NW_>), dim3(grid_wt), dim3(NW_ * 64), 0, h->stream, a); \
                               else hipLaunchKernelGGL((k_linear_mfma_wt<6, EPI, false, TPW_, 8, NW_>), dim3(grid_wt), dim3(NW_ * 64), 0, h->stream, a); } while (0)
#define EAD_LS(NW_) (rg == 7 ? launch_ls<EPI, false, NW_, 7>(h, a, grid_wt) : launch_ls<EPI, false, NW_, 8>(h, a, grid_wt))
                if (multi) { if (!EAD_LS(8)) EAD_WT(2, 4); }
                else switch (nt) {      // weight tiles straight into LDS by fetching waves; the register-ring kernel where LDS does not allow it
                    case 4: if (!EAD_LS(4)) EAD_WT(1, 4); break; case 5: if (!EAD_LS(5)) EAD_WT(1, 5); break;
                    case 6: if (!EAD_LS(6)) EAD_WT(1, 6); break; case 7: if (!EAD_LS(7)) EAD_WT(1, 7); break;
                    default: if (!EAD_LS(8)) EAD_WT(1, 8); break; }
#undef EAD_LS
#undef EAD_WT
                return;
            }
            // long passes of a matrix with few row blocks, or of a small matrix: no split of K -- a launch pair
            // per sweep would stream the matrix from memory once per sweep
            if (longpass) {
                const int sw = (TB + nt - 1) / nt, rg = rg_long, ng = (NB + rg - 1) / rg, grid_sw = (ng + 7) / 8 * 8 * sw;
                a.sweeps = sw;
                const bool ok = rg == 5 ? launch_ls<EPI, false, 8, 5>(h, a, grid_sw) : rg == 6 ? launch_ls<EPI, false, 8, 6>(h, a, grid_sw)
                              : rg == 7 ? launch_ls<EPI, false, 8, 7>(h, a, grid_sw) : launch_ls<EPI, false, 8, 8>(h, a, grid_sw);
                if (ok) return;
                a.sweeps = 0;
            }
            // one workgroup per compute unit at most: a second round would double the time
            int KS = big ? std::min(kSplitKMax, std::max(1, h->n_cu / NG)) : 1;
            while (KS > 1 && (a.K / 32) / KS < 16) --KS;
            if (KS > 1 && (size_t)KS * NG * 8 * nt * 256 <= kSplitKFloats) {
                a.KS = KS; a.sk_part = h->sk_part;
#define EAD_SK(TPW_, NW_) do { if (TPW_ != 1 || !launch_ls<EPI, true, NW_, 8>(h, a, NG * KS)) \
                                   hipLaunchKernelGGL((k_linear_mfma_wt<6, EPI, true, TPW_, 8, NW_>), dim3(NG * KS), dim3(NW_ * 64), 0, h->stream, a); \
                               hipLaunchKernelGGL((k_sk_merge<EPI, TPW_ * NW_>), dim3((NB * TPW_ * NW_ + 3) / 4), dim3(256), 0, h->stream, a, NG * 8); } while (0)
                for (a.tb_base = 0; a.tb_base < TB; a.tb_base += nt) {
                    if (multi) EAD_SK(1, 8);      // sweeps of 128 rows: eight multiplying waves, one token block each
                    else switch (nt) { case 4: EAD_SK(1, 4); break; case 5: EAD_SK(1, 5); break; case 6: EAD_SK(1, 6); break;
                                       case 7: EAD_SK(1, 7); break; default: EAD_SK(1, 8); break; }
                }
#undef EAD_SK
                return;
            }
        }
    }
    // (the rotary / cache-append epilogue is too heavy to be left to one workgroup per group)
    if (cfg == 2 && TB <= 4 && EPI != EPI_LOGITS && EPI != EPI_QKV) {
        const int NG = (NB + 3) / 4;
        int KS = std::min(kSplitKMax, std::max(1, (2 * h->n_cu + NG / 2) / NG));
        while (KS > 1 && (a.K / 32) / KS < 16) --KS;                   // a slab keeps at least 16 k tiles
        if (KS > 1 && (size_t)KS * NG * 4 * NT * 256 <= kSplitKFloats && NG <= kSplitKGroups) {
            cfg = 5; a.KS = KS; a.sk_part = h->sk_part; a.sk_tickets = h->sk_tickets; grid = NG * KS;
        }
    }
    // small matrices with few row blocks and a long K (the down projection of a narrow model: 56 row blocks,
    // 152 k tiles) leave most of the chip idle with one workgroup per row block: K is split over workgroups here
    // too, the last to arrive adds the slabs
    if constexpr (EPI == EPI_RES) {
        if (cfg == 1 && TB <= 4 && NB <= h->n_cu) {
            int KS = std::min(kSplitKMax, std::max(1, 2 * h->n_cu / NB));
            while (KS > 1 && (a.K / 32) / KS < 16) --KS;
            if (KS > 1 && (size_t)KS * NB * NT * 256 <= kSplitKFloats && NB <= kSplitKGroups) {
                cfg = 6; a.KS = KS; a.sk_part = h->sk_part; a.sk_tickets = h->sk_tickets; grid = NB * KS;
            }
        }
    }
    if (grid_cap > 0) grid = grid_cap;      // LM head: the number of partials per row is fixed
#define EAD_LM(NW_, R_, NT_, D_, SK_) hipLaunchKernelGGL((k_linear_mfma<NW_, R_, NT_, D_, EPI, SK_>), dim3(grid), dim3(NW_ * 64), 0, h->stream, a)
    switch (cfg * 10 + NT) {
        case 11: EAD_LM(4, 1, 1, 8, false); break; case 12: EAD_LM(4, 1, 2, 6, false); break; case 14: EAD_LM(4, 1, 4, 4, false); break;
        case 21: EAD_LM(8, 2, 1, 8, false); break; case 22: EAD_LM(8, 2, 2, 6, false); break; case 24: EAD_LM(8, 2, 4, 3, false); break;
        case 34: if constexpr (EPI == EPI_SWIGLU) EAD_LM(4, 2, 4, 4, false); break;
        case 41: EAD_LM(4, 4, 1, 6, false); break; case 42: EAD_LM(4, 4, 2, 4, false); break; case 44: EAD_LM(4, 4, 4, 3, false); break;
        case 51: if constexpr (EPI != EPI_LOGITS && EPI != EPI_QKV) EAD_LM(4, 4, 1, 6, true); break;
        case 52: if constexpr (EPI != EPI_LOGITS && EPI != EPI_QKV) EAD_LM(4, 4, 2, 4, true); break;
        case 54: if constexpr (EPI != EPI_LOGITS && EPI != EPI_QKV) EAD_LM(4, 4, 4, 3, true); break;
        case 61: if constexpr (EPI == EPI_RES) EAD_LM(4, 1, 1, 8, true); break;
        case 62: if constexpr (EPI == EPI_RES) EAD_LM(4, 1, 2, 6, true); break;
        default: if constexpr (EPI == EPI_RES) EAD_LM(4, 1, 4, 4, true); break;
    }
#undef EAD_LM
}

template <typename KT, int HD>
void launch_attn(ead_handle *h, int mi, AttnArgs<KT> &a, int G, int T, double kv_bytes) {
    // few rows: one workgroup per query head (latency-bound, wants the lanes); many rows:
    // one per KV head, so K and V are streamed once for the heads that share them
    const bool per_head = T <= 2 || (long)T * a.n_kv_heads * a.max_splits <= 64;
    dim3 grid(a.max_splits, per_head ? a.n_heads : a.n_kv_heads, T);
    if constexpr (std::is_same<KT, bf16_t>::value) {
        // many rows: scores and weighted sums on the matrix cores, rows of one sequence grouped
        if (!per_head && a.vtcache) {
            ProfScope ps(h, PK_ATTN, mi, kv_bytes);
#define EAD_LM_(G_) hipLaunchKernelGGL((k_attn_mfma<HD, G_>), grid, dim3(kAttnMfmaWaves * 64), 0, h->stream, a)
            switch (G) { case 1: EAD_LM_(1); break; case 2: EAD_LM_(2); break; case 3: EAD_LM_(3); break; case 4: EAD_LM_(4); break;
                         case 5: EAD_LM_(5); break; case 6: EAD_LM_(6); break; case 7: EAD_LM_(7); break; default: EAD_LM_(8); break; }
#undef EAD_LM_
            return;
        }
    }
    {
        ProfScope ps(h, PK_ATTN, mi, kv_bytes);
#define EAD_LA(G_) do { if (per_head) hipLaunchKernelGGL((k_attn<KT, HD, G_, 1>), grid, dim3(kAttnWaves * 64), 0, h->stream, a); \
                        else hipLaunchKernelGGL((k_attn<KT, HD, G_, G_>), grid, dim3(kAttnWaves * 64), 0, h->stream, a); } while (0)
        switch (G) { case 1: EAD_LA(1); break; case 2: EAD_LA(2); break; case 3: EAD_LA(3); break; case 4: EAD_LA(4); break;
                     case 5: EAD_LA(5); break; case 6: EAD_LA(6); break; case 7: EAD_LA(7); break; default: EAD_LA(8); break; }
#undef EAD_LA
    }
}

// T, n_lm, ctx_max: the host's copy of what k_plan wrote to the device plan.
template <typename WT>
ead_status forward_pass(ead_handle *h, int mi, int T, int n_lm, int ctx_max, bool dump_logits, double keys_read) {
    Model &m = h->mdl[mi];
    const int d = m.d, hd = m.hd, NQ = m.H * hd, NK = m.KV * hd, F = m.F;
    constexpr bool is_bf16 = std::is_same<WT, bf16_t>::value;
    const bool mfma = is_bf16 && T > 2;      // the FMA path takes 1, 2 or 4 rows a pass and is slow at 4
    hipStream_t st = h->stream;
    const int *cnt = h->plan.hdr;
    const int T16 = (T + 15) & ~15;

    {
        ProfScope ps(h, PK_EMBED, mi, 0.0);
        hipLaunchKernelGGL(k_embed<WT>, dim3(T), dim3(256), 0, st, (const WT *)m.embed, h->s.tokens, cnt, h->plan.row_seq,
                           h->plan.row_pos, h->s.max_seq, d, h->x);
    }
    const double attn_bytes = keys_read * 2.0 * NK * sizeof(WT);
    // attention split: a workgroup (8 waves) takes at least 512 keys; more splits only while
    // that helps to fill the chip, never more than 16 (the last one merges them all), bounded scratch
    // (a decode step of one or two rows is a chain of latencies: splits of 128 keys, one workgroup per
    // query head and split, spread it over more compute units: +3 % tokens/s at batch 1 against 512)
    int chunk = T <= 2 ? 128 : 512;
    while ((long)T * m.KV * ((ctx_max + chunk - 1) / chunk) > 1024 && chunk < 65536) chunk <<= 1;
    while ((ctx_max + chunk - 1) / chunk > kAttnMaxSplits) chunk <<= 1;
    while ((long)T * ((ctx_max + chunk - 1) / chunk) > h->items_max) chunk <<= 1;
    // the matrix-core kernel (many rows) is bound by the latency of its short chains of loads, two
    // workgroups per compute unit at a time: fewer, longer workgroups
    if (is_bf16 && m.layers[0].vtcache && T > 2 && (long)T * m.KV * ((ctx_max + chunk - 1) / chunk) > 64)
        while ((long)T * m.KV * ((ctx_max + chunk - 1) / chunk) > 2 * h->n_cu && chunk < 65536) chunk <<= 1;
    const int max_splits = (ctx_max + chunk - 1) / chunk;

    for (int l = 0; l < m.L; ++l) {
        Layer &ly = m.layers[l];
        // ---- RMSNorm + QKV + rotary + KV append ----
        LinArgs<WT> a{};
        a.W = (const WT *)ly.wqkv; a.Np = NQ + 2 * NK; a.K = d; a.count = cnt; a.out = h->q; a.ldo = NQ;
        a.kcache = (WT *)ly.kcache; a.vcache = (WT *)ly.vcache; a.vtcache = (WT *)ly.vtcache; a.row_seq = h->plan.row_seq; a.row_pos = h->plan.row_pos;
        a.rope = m.rope; a.n_heads = m.H; a.n_kv_heads = m.KV; a.hd = hd; a.max_seq = h->s.max_seq;
        if (mfma) {
            if constexpr (is_bf16) {
                PackArgs pa{h->x, d, cnt, nullptr, ly.g_attn, m.eps, h->xp_a, d};
                { ProfScope ps(h, PK_PACK_ACT, mi, 0.0); hipLaunchKernelGGL(k_pack_act, dim3(T16), dim3(256), 0, st, pa); }
                a.xp = h->xp_a;
                launch_mfma<EPI_QKV>(h, mi, a, T);
            }
        } else {
            a.x = h->x; a.ldx = d; a.gain = ly.g_attn; a.eps = m.eps;
            launch_valu<WT, EPI_QKV>(h, mi, a, T, a.Np / 16);
        }
        // ---- attention ----
        AttnArgs<WT> at{};
        at.q = h->q; at.kcache = (const WT *)ly.kcache; at.vcache = (const WT *)ly.vcache; at.vtcache = (const WT *)ly.vtcache; at.count = cnt;
        at.row_seq = h->plan.row_seq; at.row_pos = h->plan.row_pos; at.n_heads = m.H; at.n_kv_heads = m.KV;
        at.max_seq = h->s.max_seq; at.chunk = chunk; at.max_splits = max_splits; at.scale = 1.0f / sqrtf((float)hd);
        at.part_o = h->part_o; at.part_ml = h->part_ml; at.tickets = h->tickets;
        if (mfma) at.out_tiles = h->xp_o; else at.out = h->o;
        if (h->attn_order_n == T) { at.use_order = 1; memcpy(at.order, h->attn_order, (size_t)T); }
        if (hd == 32) launch_attn<WT, 32>(h, mi, at, m.H / m.KV, T, attn_bytes);
        else if (hd == 64) launch_attn<WT, 64>(h, mi, at, m.H / m.KV, T, attn_bytes);
        else launch_attn<WT, 128>(h, mi, at, m.H / m.KV, T, attn_bytes);
        // ---- output projection + residual ----
        LinArgs<WT> b{};
        b.W = (const WT *)ly.wo; b.Np = d; b.K = NQ; b.count = cnt; b.out = h->x; b.ldo = d;
        if (mfma) { if constexpr (is_bf16) { b.xp = h->xp_o; launch_mfma<EPI_RES>(h, mi, b, T); } }
        else { b.x = h->o; b.ldx = NQ; launch_valu<WT, EPI_RES>(h, mi, b, T, d / 16); }
        // ---- RMSNorm + gate/up + SwiGLU ----
        LinArgs<WT> c{};
        c.W = (const WT *)ly.wgu; c.Np = 2 * F; c.K = d; c.count = cnt; c.ldo = F;
        if (mfma) {
            if constexpr (is_bf16) {
                PackArgs pa{h->x, d, cnt, nullptr, ly.g_ffn, m.eps, h->xp_a, d};
                { ProfScope ps(h, PK_PACK_ACT, mi, 0.0); hipLaunchKernelGGL(k_pack_act, dim3(T16), dim3(256), 0, st, pa); }
                c.xp = h->xp_a; c.out_tiles = h->xp_h; c.tbs = T16 / 16;
                launch_mfma<EPI_SWIGLU>(h, mi, c, T);
            }
        } else {
            c.x = h->x; c.ldx = d; c.gain = ly.g_ffn; c.eps = m.eps; c.out = h->hbuf;
            // two resident workgroups per CU stride over the row blocks: activations are staged once
            launch_valu<WT, EPI_SWIGLU>(h, mi, c, T, std::min(c.Np / 16, 2 * h->n_cu));
        }
        // ---- down projection + residual ----
        LinArgs<WT> e{};
        e.W = (const WT *)ly.wdown; e.Np = d; e.K = F; e.count = cnt; e.out = h->x; e.ldo = d;
        if (mfma) { if constexpr (is_bf16) { e.xp = h->xp_h; launch_mfma<EPI_RES>(h, mi, e, T); } }
        else { e.x = h->hbuf; e.ldx = F; launch_valu<WT, EPI_RES>(h, mi, e, T, d / 16); }
    }
    if (n_lm > 0) {
        // ---- final RMSNorm + LM head with the entropy statistics folded in ----
        LinArgs<WT> g{};
        g.W = (const WT *)m.lm_head; g.Np = m.V; g.K = d; g.count = cnt + 1; g.rowmap = h->plan.lm_row;
        g.partials = h->lm_part; g.logits = dump_logits ? h->logits_dump : nullptr;
        if (h->samp_temp > 0.f && !h->scoring) {
            g.samp_inv_t = 1.0f / h->samp_temp; g.samp_k0 = (uint32_t)h->samp_seed; g.samp_k1 = (uint32_t)(h->samp_seed >> 32);
            g.samp_seq = h->plan.lm_seq; g.samp_ngen = h->s.ngen;
        }
        const int grid = std::min(m.V / 16, h->lm_grid);
        if (is_bf16 && n_lm > 2) {
            if constexpr (is_bf16) {
                PackArgs pa{h->x, d, cnt + 1, h->plan.lm_row, m.g_final, m.eps, h->xp_a, d};
                { ProfScope ps(h, PK_PACK_ACT, mi, 0.0); hipLaunchKernelGGL(k_pack_act, dim3((n_lm + 15) & ~15), dim3(256), 0, st, pa); }
                g.xp = h->xp_a;
                launch_mfma<EPI_LOGITS>(h, mi, g, n_lm, grid);
            }
        } else {
            g.x = h->x; g.ldx = d; g.gain = m.g_final; g.eps = m.eps;
            launch_valu<WT, EPI_LOGITS>(h, mi, g, n_lm, grid);
        }
    }
    HIP_TRY(h, hipGetLastError());
    return EAD_OK;
}

// keys read by the pass the host just planned (kvlen not yet advanced): row j of a sequence
// that had `have` positions reads have + j + 1 keys
double keys_in_pass(ead_handle *h, int mi, const std::vector<int> &rows) {
    double k = 0.0;
    for (int b = 0; b < h->batch; ++b)
        if (rows[b]) k += (double)rows[b] * h->hs[b].kvlen[mi] + (double)rows[b] * (rows[b] + 1) / 2.0;
    return k;
}

ead_status run_pass(ead_handle *h, int mi, int T, int n_lm, int ctx_max, bool dump, const std::vector<int> &rows) {
    const double keys = keys_in_pass(h, mi, rows);
    // the pass's rows by falling context (plan order: sequences in index order, a sequence's rows in a row)
    h->attn_order_n = 0;
    if (T > 2 && T <= kAttnOrderMax) {
        std::pair<int, int> pr[kAttnOrderMax];      // (position, row)
        int t = 0;
        for (int b = 0; b < h->batch; ++b)
            for (int i = 0; i < rows[b]; ++i, ++t) pr[t] = {h->hs[b].kvlen[mi] + i, t};
        if (t == T) {
            std::stable_sort(pr, pr + T, [](const std::pair<int, int> &x, const std::pair<int, int> &y) { return x.first > y.first; });
            for (int i = 0; i < T; ++i) h->attn_order[i] = (unsigned char)pr[i].second;
            h->attn_order_n = T;
        }
    }
    return h->mdl[mi].dtype == EAD_BF16 ? forward_pass<bf16_t>(h, mi, T, n_lm, ctx_max, dump, keys)
                                        : forward_pass<float>(h, mi, T, n_lm, ctx_max, dump, keys);
}

// ---- fused single-row decode step ---------------------------------------------------------
template <typename WT, int HD, int G>
void *fused_kernel_ptr() { return (void *)k_decode_fused<WT, HD, G>; }

// the (dtype, head_dim, heads per KV head) combinations the fused kernel is built for
void *fused_kernel_for(const Model &m) {
    const int G = m.H / m.KV;
    if (m.dtype == EAD_F32) {
        if (m.hd == 32 && G == 1) return fused_kernel_ptr<float, 32, 1>();
        if (m.hd == 32 && G == 2) return fused_kernel_ptr<float, 32, 2>();
        return nullptr;
    }
    if (m.hd == 64 && G == 4) return fused_kernel_ptr<bf16_t, 64, 4>();
    if (m.hd == 128 && G == 4) return fused_kernel_ptr<bf16_t, 128, 4>();
    if (m.hd == 64 && G == 7) return fused_kernel_ptr<bf16_t, 64, 7>();
    if (m.hd == 128 && G == 5) return fused_kernel_ptr<bf16_t, 128, 5>();
    return nullptr;
}

// the streamed variant: bf16 only
template <int HD, int G>
void *stream_kernel_ptr() { return (void *)k_decode_stream<HD, G>; }
void *stream_kernel_for(const Model &m) {
    const int G = m.H / m.KV;
    if (m.dtype != EAD_BF16) return nullptr;
    if (m.hd == 64 && G == 4) return stream_kernel_ptr<64, 4>();
    if (m.hd == 128 && G == 4) return stream_kernel_ptr<128, 4>();
    if (m.hd == 64 && G == 7) return stream_kernel_ptr<64, 7>();
    if (m.hd == 128 && G == 5) return stream_kernel_ptr<128, 5>();
    return nullptr;
}
size_t stream_lds_bytes(const Model &m) {
    const size_t kmax = std::max(std::max(m.d, m.F), m.H * m.hd);
    const size_t attn = (size_t)kFusedWaves * m.hd + 2 * kFusedWaves;
    return (size_t)kStreamDepth * kStreamSlotBytes + std::max(kmax + 2 * kFusedWaves * 16 + 64, attn) * sizeof(float);
}

size_t fused_lds_bytes(const Model &m) {
    const size_t kmax = std::max(std::max(m.d, m.F), m.H * m.hd);
    const size_t G = m.H / m.KV;
    const size_t attn = (size_t)kFusedWaves * m.hd + 2 * kFusedWaves + 0 * G;
    return std::max(kmax + (size_t)kFusedRbChunk * kFusedWaves * 16 + 64, attn) * sizeof(float);
}

FinArgs make_fin(ead_handle *h, int m, bool score) {
    FinArgs fa{};
    fa.s = h->s; fa.p = h->plan; fa.cfg = h->cfg; fa.partials = h->lm_part;
    fa.n_part = std::min(h->mdl[m].V / 16, h->lm_grid); fa.unit = h->prm.unit;
    fa.score_mode = score ? 1 : 0; fa.sc_H = h->sc_H; fa.sc_arg = h->sc_arg;
    fa.model_id = m; fa.max_new = h->max_new; fa.eos_id = h->prm.eos_id; fa.replay = h->replay; fa.n_new = h->n_new;
    fa.force_model = h->force_model; fa.step = h->step;
    fa.sampling = (!score && h->samp_temp > 0.f) ? 1 : 0;
    fa.host_model = h->lanes[0].rb_model; fa.host_done = h->lanes[0].rb_done;      // one array for both lanes: entries are per sequence
    return fa;
}

template <typename WT>
ead_status fused_step(ead_handle *h, int mi, double keys) {
    Model &m = h->mdl[mi];
    FusedArgs<WT> a{};
    a.L = m.L; a.d = m.d; a.H = m.H; a.KV = m.KV; a.hd = m.hd; a.F = m.F; a.V = m.V; a.eps = m.eps;
    a.mats = (const FusedMat<WT> *)m.fused_mats; a.layers = (const FusedLayer<WT> *)m.fused_layers; a.n_mats = m.n_mats;
    a.embed = (const WT *)m.embed; a.g_final = m.g_final; a.rope = m.rope;
    a.x = h->x; a.q = h->q; a.hbuf = h->hbuf; a.att_o = h->att_o; a.att_ml = h->att_ml; a.lm_part = h->lm_part;
    a.bar = GridBar{h->bar_mem, h->bar_mem + kBarGroups * 32, h->abort_flag, h->bar_epoch};
    a.fin = make_fin(h, mi, false);
    a.batch = h->batch;
    ProfScope ps(h, PK_FUSED, mi, m.weight_bytes_nolm + m.lm_bytes + keys * m.kv_bytes_per_pos);
    if constexpr (std::is_same<WT, bf16_t>::value) {
        if (m.stream_ok && h->fused_on != 2) {
            StreamModel sm{};
            const int NQ = m.H * m.hd, NK = m.KV * m.hd;
            sm.base = (const bf16_t *)m.arena; sm.layer_stride = m.layer_elems; sm.lm = (const bf16_t *)m.lm_head; sm.L = m.L;
            for (int j = 0; j < 4; ++j) sm.off[j] = m.mat_off[j];
            sm.NB[0] = (NQ + 2 * NK) / 16; sm.KC[0] = m.d / 32;
            sm.NB[1] = m.d / 16; sm.KC[1] = NQ / 32;
            sm.NB[2] = 2 * m.F / 16; sm.KC[2] = m.d / 32;
            sm.NB[3] = m.d / 16; sm.KC[3] = m.F / 32;
            sm.NB[4] = m.V / 16; sm.KC[4] = m.d / 32;
            void *sargs[] = {&a, &sm};
            HIP_TRY(h, hipLaunchCooperativeKernel(stream_kernel_for(m), dim3(h->fused_grid), dim3(kStreamThreads), sargs,
                                                  (unsigned)stream_lds_bytes(m), h->stream));
            h->bar_epoch += 5u * m.L + 1u;
            return EAD_OK;
        }
    }
    void *args[] = {&a};
    HIP_TRY(h, hipLaunchCooperativeKernel(fused_kernel_for(m), dim3(h->fused_grid), dim3(kFusedThreads), args,
                                          (unsigned)fused_lds_bytes(m), h->stream));
    h->bar_epoch += 5u * m.L + 1u;
    return EAD_OK;
}

// Host copy of k_plan: which rows the pass will hold.  Returns T; fills n_lm, ctx_max and,
// per sequence, how many rows it got and whether its chunk reaches the end.
int host_plan(ead_handle *h, int m, int budget, int limit_off, int lm_mode, bool ignore_model, int step, int *n_lm,
              int *ctx_max, std::vector<int> *rows, std::vector<char> *complete) {
    int off = 0, nlm = 0, cm = 0;
    rows->assign(h->batch, 0); complete->assign(h->batch, 0);
    for (int b = 0; b < h->batch; ++b) {
        HostSeq &s = h->hs[b];
        const bool active = !s.done && (ignore_model || s.model == m) && (step < 0 || s.last_step != step) &&
                            (ignore_model || s.ngen < s.goal);
        const int target = s.len - limit_off, have = s.kvlen[m];
        int n = active ? std::max(0, target - have) : 0;
        n = std::min(n, budget - off);
        (*rows)[b] = n;
        if (n > 0) {
            cm = std::max(cm, have + n);
            if (have + n == target) { (*complete)[b] = 1; if (lm_mode == 1) ++nlm; }
        }
        off += n;
    }
    *n_lm = lm_mode == 2 ? off : nlm;
    *ctx_max = cm;
    return off;
}

void launch_plan(ead_handle *h, int m, int budget, int limit_off, int lm_mode, bool ignore_model, int step,
                 const std::vector<int> *rows = nullptr) {
    PlanArgs pa{h->s, h->plan, h->batch, m, budget, limit_off, lm_mode, ignore_model ? 1 : 0, step, 0, {0}};
    if (rows && h->two_lanes) {          // name the sequences of this pass (see PlanArgs)
        pa.use_allow = 1;
        for (int b = 0; b < h->batch; ++b) if ((*rows)[b] > 0) pa.allow[b >> 6] |= 1ull << (b & 63);
    }
    ProfScope ps(h, PK_PLAN, m, 0.0);
    hipLaunchKernelGGL(k_plan, dim3(1), dim3(256), 3 * h->batch * sizeof(int), h->stream, pa);
}

void launch_finalize(ead_handle *h, int m, int n_lm, bool score) {
    FinArgs fa = make_fin(h, m, score);
    ProfScope ps(h, PK_FINALIZE, m, 0.0);
    hipLaunchKernelGGL(k_lm_finalize, dim3(n_lm), dim3(64), 0, h->stream, fa);
}

void account_pass(ead_handle *h, int m, const std::vector<int> &rows, bool with_lm) {
    Model &md = h->mdl[m];
    h->stats.algorithmic_bytes += md.weight_bytes_nolm + (with_lm ? md.lm_bytes : 0.0) +
                                  md.kv_bytes_per_pos * keys_in_pass(h, m, rows);
}

ead_status validate_prompts(ead_handle *h, const int32_t *toks, const int32_t *lens, int batch, int max_new) {
    if (!toks || !lens) return fail(h, EAD_ERR_INVALID_ARG, "null prompt pointer");
    if (batch < 1 || max_new < 1) return fail(h, EAD_ERR_INVALID_ARG, "batch and max_new_tokens must be >= 1");
    if (batch > h->prm.max_batch) return fail(h, EAD_ERR_SEQ_OVERFLOW, "batch %d exceeds max_batch %d", batch, h->prm.max_batch);
    if (max_new > h->prm.max_seq) return fail(h, EAD_ERR_SEQ_OVERFLOW, "max_new_tokens %d exceeds max_seq %d", max_new, h->prm.max_seq);
    size_t off = 0;
    for (int b = 0; b < batch; ++b) {
        if (lens[b] < 1) return fail(h, EAD_ERR_INVALID_ARG, "prompt %d is empty", b);
        if ((long)lens[b] + max_new > h->prm.max_seq)
            return fail(h, EAD_ERR_SEQ_OVERFLOW, "prompt %d: %d + %d tokens exceed max_seq %d", b, lens[b], max_new, h->prm.max_seq);
        for (int i = 0; i < lens[b]; ++i)
            if (toks[off + i] < 0 || toks[off + i] >= h->mdl[0].V)
                return fail(h, EAD_ERR_INVALID_ARG, "prompt %d token %d out of range", b, i);
        off += lens[b];
    }
    return EAD_OK;
}

// Algorithm 1's initialisation for every sequence of the run (W empty, M = M_S, c = 0, nothing generated),
// on the host mirror and on the device.  kv_fill = 0: no model has consumed anything yet (ead_begin, before
// the prompt passes); 1: both models hold every prompt position but the last (ead_rewind).
ead_status reset_run_state(ead_handle *h, int max_new, int kv_fill) {
    hipStream_t st = h->stream;
    const int MB = h->s.max_batch, batch = h->batch;
    h->max_new = max_new; h->began = 0; h->step = 0; h->sched_phase = 0;
    h->hs.assign(batch, HostSeq{});
    std::vector<int> len(MB, 0), zeros(MB * 2, 0), kv(MB * 2, 0), model(MB, 0), neg(MB, -1), goal(MB, max_new);
    for (int b = 0; b < batch; ++b) {
        HostSeq &s = h->hs[b];
        s.len = len[b] = h->prompt_len[b];
        s.kvlen[0] = s.kvlen[1] = kv[b] = kv[MB + b] = kv_fill ? h->prompt_len[b] - 1 : 0;
        s.c = 0; s.ngen = 0; s.done = 0; s.last_step = -1; s.goal = max_new;
        s.model = h->force_model >= 0 ? h->force_model : (h->replay ? -1 : 0);
        model[b] = std::max(s.model, 0);
    }
    HIP_TRY(h, hipMemcpyAsync(h->s.len, len.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.kvlen, kv.data(), 2 * MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.model, model.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.c, zeros.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.ngen, zeros.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.done, zeros.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.last_step, neg.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.goal, goal.data(), MB * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.err, zeros.data(), sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipStreamSynchronize(st));          // the staging vectors leave scope
    return EAD_OK;
}

ead_status begin_impl(ead_handle *h, const int32_t *toks, const int32_t *lens, int batch, int max_new) {
    use_lane(h, 0);
    if (h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1].stream));
    TRY(validate_prompts(h, toks, lens, batch, max_new));
    hipStream_t st = h->stream;
    const int MS = h->s.max_seq;
    h->batch = batch; h->prefilled = 0;
    h->prompt_len.assign(lens, lens + batch);
    std::vector<int> tok((size_t)batch * MS, 0);
    size_t off = 0;
    for (int b = 0; b < batch; ++b) {
        memcpy(&tok[(size_t)b * MS], toks + off, sizeof(int) * lens[b]);
        off += lens[b];
    }
    HIP_TRY(h, hipMemcpyAsync(h->s.tokens, tok.data(), tok.size() * sizeof(int), hipMemcpyHostToDevice, st));
    TRY(reset_run_state(h, max_new, 0));           // waits for the stream: tok may leave scope
    // both models consume every prompt token but the last
    std::vector<int> rows; std::vector<char> complete;
    for (int m = 0; m < 2; ++m) {
        for (;;) {
            int n_lm, ctx_max;
            const int T = host_plan(h, m, h->Tmax, 1, 0, true, -1, &n_lm, &ctx_max, &rows, &complete);
            if (T == 0) break;
            launch_plan(h, m, h->Tmax, 1, 0, true, -1);
            TRY(run_pass(h, m, T, 0, ctx_max, false, rows));
            for (int b = 0; b < batch; ++b) h->hs[b].kvlen[m] += rows[b];
        }
    }
    HIP_TRY(h, hipStreamSynchronize(st));
    memset(&h->stats, 0, sizeof h->stats);
    h->began = 1;
    h->prefilled = h->replay ? 0 : 1;
    return EAD_OK;
}

// One forward pass of model m over the rows the plan gives it, with the host's copy of
// the per-sequence state advanced for the rows that produced a token.  Returns the number of
// token rows through *T_out (0: nothing to do).  `step` gates rows that already produced a
// token in this lock-step iteration; -1 takes every eligible row.
ead_status decode_pass(ead_handle *h, int m, int step, std::vector<char> &emitted, int *T_out) {
    std::vector<int> rows; std::vector<char> complete;
    int n_lm, ctx_max;
    const int T = host_plan(h, m, h->Tmax, 0, 1, false, step, &n_lm, &ctx_max, &rows, &complete);
    *T_out = T;
    if (T == 0) return EAD_OK;
    if (T == 1 && n_lm == 1 && h->batch == 1 && h->fused_on && h->mdl[m].fused_ok && !(h->samp_temp > 0.f)) {
        const double keys = keys_in_pass(h, m, rows);
        TRY(h->mdl[m].dtype == EAD_BF16 ? fused_step<bf16_t>(h, m, keys) : fused_step<float>(h, m, keys));
    } else {
        launch_plan(h, m, h->Tmax, 0, 1, false, step, &rows);
        TRY(run_pass(h, m, T, n_lm, ctx_max, false, rows));
        if (n_lm > 0) launch_finalize(h, m, n_lm, false);
    }
    account_pass(h, m, rows, n_lm > 0);
    if (n_lm > 0) (m ? h->stats.steps_large : h->stats.steps_small)++;
    for (int b = 0; b < h->batch; ++b) {
        HostSeq &s = h->hs[b];
        if (!rows[b]) continue;
        const int extra = rows[b] - (complete[b] ? 1 : 0);
        (m ? h->stats.catchup_rows_large : h->stats.catchup_rows_small) += extra;
        s.kvlen[m] += rows[b];
        if (complete[b]) {
            emitted[b] = 1; s.last_step = step;
            (m ? h->stats.tokens_large : h->stats.tokens_small)++;
        }
    }
    return EAD_OK;
}

// Advance the host's copy of the state of the rows that produced a token, and learn from the
// device which model serves them next -- only when that can have changed (a row's counter has
// reached d_min, or an end-of-sequence id can end it).
// The read-back goes through the current lane's stream; all_lanes: rows of both lanes produced
// tokens (lock step), so the other lane's stream is waited for first.
ead_status after_tokens(ead_handle *h, const std::vector<char> &emitted, bool all_lanes) {
    LaneSet &ln = h->lanes[h->cur_lane];
    hipStream_t st = ln.stream;
    int *rb_model = h->lanes[0].rb_model, *rb_done = h->lanes[0].rb_done;
    bool need_sync = h->prm.eos_id >= 0;
    for (int b = 0; b < h->batch; ++b) {
        if (!emitted[b]) continue;
        HostSeq &s = h->hs[b];
        s.len++; s.ngen++; s.c++;
        if (s.ngen >= h->max_new) s.done = 1;
        if (h->replay || h->force_model >= 0) continue;
        if (s.c >= h->cfg.d_min && !s.done) need_sync = true;
    }
    if (h->replay) {
        // the next model is dictated: read it from the host copy of the forced ids
        for (int b = 0; b < h->batch; ++b) {
            HostSeq &s = h->hs[b];
            if (!emitted[b] || s.done) continue;
            const int nxt = h->h_model[(size_t)b * h->s.cap + s.ngen];   // forced ids staged by ead_replay
            if (nxt != s.model) { s.model = nxt; s.c = 0; h->stats.switches++; }
        }
    } else if (need_sync && h->force_model < 0) {
        if (all_lanes && h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1 - h->cur_lane].stream));
        HIP_TRY(h, hipStreamSynchronize(st));      // the pass's last kernel wrote rb_model / rb_done (pinned) itself
        h->stats.host_syncs++;
        for (int b = 0; b < h->batch; ++b) {
            HostSeq &s = h->hs[b];
            if (!emitted[b]) continue;              // entries of rows in flight on the other lane are not at rest
            if (rb_done[b]) s.done = 1;
            if (rb_model[b] != s.model) { s.model = rb_model[b]; s.c = 0; h->stats.switches++; }
        }
    } else if (need_sync) {
        if (all_lanes && h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1 - h->cur_lane].stream));
        HIP_TRY(h, hipStreamSynchronize(st));
        for (int b = 0; b < h->batch; ++b) if (emitted[b] && rb_done[b]) h->hs[b].done = 1;
    }
    return EAD_OK;
}

// Grouped schedule.  Every sequence is its own instance of Algorithm 1, so rows need not move
// in lock step: rows served by the small model run ahead through cheap small passes while rows
// that switched to the large model wait, and one large pass then serves all that have
// gathered -- the large model's weights are streamed once for many rows instead of once per
// token position.  The large model starts running when at least `hi` of the unfinished rows
// wait for it and keeps running until fewer than `lo` do (rows stay on it for at least d_min
// tokens, so its passes come in bursts).  No row's arithmetic depends on the schedule.
// budget < 0: every row produces up to n_tokens more tokens (per-sequence goals).  budget >= 0: the batch as a
// whole produces at least `budget` more tokens; rows run freely, none more than `lead` tokens ahead of the
// unfinished row that has produced the fewest, and no pass is started once the budget is met.
ead_status decode_grouped(ead_handle *h, int n_tokens, long budget = -1, int lead = 0) {
    use_lane(h, 0);
    hipStream_t st = h->stream;
    std::vector<int> goal(h->s.max_batch, 0);
    const bool by_budget = budget >= 0;
    const long produced0 = h->stats.tokens_small + h->stats.tokens_large;
    auto exhausted = [&]() { return by_budget && h->stats.tokens_small + h->stats.tokens_large - produced0 >= budget; };
    // budget mode: the host's copy of the goals follows the slowest row; the device's stay at the bound of the
    // run, and every pass names its sequences to the plan kernel
    auto update_goals = [&]() {
        if (!by_budget) return;
        int lo = h->max_new;
        for (int b = 0; b < h->batch; ++b) if (!h->hs[b].done) lo = std::min(lo, h->hs[b].ngen);
        for (int b = 0; b < h->batch; ++b) h->hs[b].goal = (int)std::min<long>(h->max_new, (long)lo + lead);
    };
    if (!by_budget) {
        for (int b = 0; b < h->batch; ++b) {
            HostSeq &s = h->hs[b];
            s.goal = (int)std::min<long>(h->max_new, (long)s.ngen + n_tokens);
            goal[b] = s.goal;
        }
        HIP_TRY(h, hipMemcpyAsync(h->s.goal, goal.data(), h->s.max_batch * sizeof(int), hipMemcpyHostToDevice, st));
        HIP_TRY(h, hipStreamSynchronize(st));      // `goal` leaves scope; the other lane starts after this too
    }
    auto waiting = [&](int n[2]) {
        update_goals();
        n[0] = n[1] = 0;
        if (exhausted()) return;
        for (int b = 0; b < h->batch; ++b) {
            const HostSeq &s = h->hs[b];
            if (!s.done && s.ngen < s.goal) n[s.model ? 1 : 0]++;
        }
    };
    if (!h->two_lanes) {
        // one pass at a time: the small model while the large one gathers rows, then the large one
        std::vector<char> emitted(h->batch);
        for (;;) {
            int n[2];
            waiting(n);
            const int N = n[0] + n[1];
            if (N == 0) break;
            if (n[1] == 0) h->sched_phase = 0;
            else if (n[0] == 0) h->sched_phase = 1;
            else if (h->sched_phase == 1 && (float)n[1] < h->sched_lo * (float)N) h->sched_phase = 0;
            else if (h->sched_phase == 0 && (float)n[1] >= h->sched_hi * (float)N) h->sched_phase = 1;
            const int m = h->sched_phase;
            std::fill(emitted.begin(), emitted.end(), 0);
            int T = 0;
            TRY(decode_pass(h, m, -1, emitted, &T));
            if (T == 0) return fail(h, EAD_ERR_STATE, "scheduler found no work for model %d", m);
            TRY(after_tokens(h, emitted, false));
            h->step++;
        }
    } else {
        // Two lanes: the small model's passes (bound by latency) and the large model's (bound by
        // bandwidth) run side by side on their own streams and scratch.  A lane takes a new pass
        // as soon as its last one has been read back; rows change lanes when the host has seen
        // their switch.  The large lane still waits until enough rows have gathered.
        std::vector<char> em[2] = {std::vector<char>(h->batch), std::vector<char>(h->batch)};
        bool busy[2] = {false, false};
        int small_held = 0;                           // times in a row the small lane was held back while it had rows
        for (;;) {
            int n[2];
            waiting(n);                               // rows of a busy lane count as waiting for it: they are in its pass
            const int N = n[0] + n[1];
            if (N == 0 && !busy[0] && !busy[1]) break;
            if (!busy[1]) {
                if (n[1] == 0) h->sched_phase = 0;
                else if (n[0] == 0 && !busy[0]) h->sched_phase = 1;
                else if (h->sched_phase == 1 && (float)n[1] < h->sched_lo * (float)N) h->sched_phase = 0;
                else if (h->sched_phase == 0 && (float)n[1] >= h->sched_hi * (float)N) h->sched_phase = 1;
            }
            for (int m = 1; m >= 0; --m) {
                if (busy[m] || n[m] == 0 || (m == 1 && h->sched_phase != 1)) continue;
                // a small pass costs the same 170 launches for 5 rows as for 50 and slows the
                // large pass beside it: while the large lane is busy the small lane waits until
                // kSmallLaneMin of the unfinished rows are ready for it
                // (for at most two large passes in a row, so that a few small-model rows are not left
                // behind while the large lane serves burst after burst)
                if (m == 0 && busy[1] && (float)n[0] < kSmallLaneMin * (float)N && small_held < 2) {
                    ++small_held;
                    continue;
                }
                if (m == 0) small_held = 0;
                use_lane(h, m);
                std::fill(em[m].begin(), em[m].end(), 0);
                int T = 0;
                TRY(decode_pass(h, m, -1, em[m], &T));
                if (T == 0) return fail(h, EAD_ERR_STATE, "scheduler found no work for model %d", m);
                HIP_TRY(h, hipEventRecord(h->lanes[m].done_ev, h->lanes[m].stream));
                busy[m] = true;
            }
            if (!busy[0] && !busy[1]) return fail(h, EAD_ERR_STATE, "scheduler stalled with %d rows waiting", N);
            // whichever lane finishes first is read back first
            int fin = -1;
            if (busy[0] && busy[1]) {
                for (;;) {
                    hipError_t q0 = hipEventQuery(h->lanes[0].done_ev);
                    if (q0 == hipSuccess) { fin = 0; break; }
                    if (q0 != hipErrorNotReady) HIP_TRY(h, q0);
                    hipError_t q1 = hipEventQuery(h->lanes[1].done_ev);
                    if (q1 == hipSuccess) { fin = 1; break; }
                    if (q1 != hipErrorNotReady) HIP_TRY(h, q1);
                }
            } else {
                fin = busy[0] ? 0 : 1;
                HIP_TRY(h, hipEventSynchronize(h->lanes[fin].done_ev));
            }
            use_lane(h, fin);
            TRY(after_tokens(h, em[fin], false));
            busy[fin] = false;
            h->step++;
        }
        use_lane(h, 0);
    }
    // pauses end here: rows may run to the bound of the run again
    for (int b = 0; b < h->batch; ++b) { h->hs[b].goal = h->max_new; goal[b] = h->max_new; }
    if (!by_budget) {
        HIP_TRY(h, hipMemcpyAsync(h->s.goal, goal.data(), h->s.max_batch * sizeof(int), hipMemcpyHostToDevice, st));
        HIP_TRY(h, hipStreamSynchronize(st));
    }
    return EAD_OK;
}

ead_status decode_impl(ead_handle *h, int n_steps, long budget = -1, int lead = 0) {
    if (!h->began) return fail(h, EAD_ERR_STATE, "ead_decode before ead_begin");
    use_lane(h, 0);
    hipStream_t st = h->stream;
    std::vector<char> emitted(h->batch);
    if (h->sched_grouped || budget >= 0) {
        TRY(decode_grouped(h, n_steps, budget, lead));
        n_steps = 0;
    }
    bool used_prev[2] = {false, false};
    for (int it = 0; it < n_steps; ++it) {
        const int step = h->step;
        std::fill(emitted.begin(), emitted.end(), 0);
        bool any = false;
        // The two models serve disjoint rows: their passes go to two streams and run side by side.
        // A row may change lanes from one step to the next without the host having waited (its
        // next model can be known in advance), so a lane first waits for the other lane's
        // previous step; the passes of one step still overlap.
        bool used[2] = {false, false};
        for (int m = 0; m < 2; ++m) {
            use_lane(h, m);
            for (;;) {
                std::vector<int> probe_rows; std::vector<char> probe_complete;
                int n_lm = 0, ctx_max = 0;
                if (h->two_lanes && !used[m] && used_prev[1 - m] &&
                    host_plan(h, m, h->Tmax, 0, 1, false, step, &n_lm, &ctx_max, &probe_rows, &probe_complete) > 0)
                    HIP_TRY(h, hipStreamWaitEvent(h->lanes[m].stream, h->lanes[1 - m].done_ev, 0));
                int T = 0;
                TRY(decode_pass(h, m, step, emitted, &T));
                if (T == 0) break;
                any = true; used[m] = true;
            }
        }
        if (h->two_lanes)
            for (int m = 0; m < 2; ++m)
                if (used[m]) HIP_TRY(h, hipEventRecord(h->lanes[m].done_ev, h->lanes[m].stream));
        used_prev[0] = used[0]; used_prev[1] = used[1];
        use_lane(h, 0);
        if (!any) break;
        TRY(after_tokens(h, emitted, true));
        h->step++;
    }
    if (h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1].stream));
    HIP_TRY(h, hipStreamSynchronize(st));
    int err = 0, aborted = 0;
    HIP_TRY(h, hipMemcpy(&aborted, h->abort_flag, sizeof(int), hipMemcpyDeviceToHost));
    if (aborted) {
        // a grid barrier gave up: drop the fused path for this handle and start its counters afresh
        h->fused_on = 0; h->bar_epoch = 0; h->began = 0;
        HIP_TRY(h, hipMemset(h->bar_mem, 0, (kBarGroups * 32 + 32) * sizeof(unsigned)));
        HIP_TRY(h, hipMemset(h->abort_flag, 0, sizeof(int)));
        return fail(h, EAD_ERR_DEVICE, "fused decode kernel abandoned a grid barrier; fused path disabled, run again");
    }
    HIP_TRY(h, hipMemcpy(&err, h->s.err, sizeof(int), hipMemcpyDeviceToHost));
    if (err) return fail(h, EAD_ERR_NONFINITE, "a non-finite entropy was produced (non-finite logits)");
    return EAD_OK;
}

ead_status fetch_impl(ead_handle *h, int stride, int32_t *tok, uint8_t *mid, float *H, float *Hbar, uint8_t *dec,
                      int32_t *lens) {
    if (!h->began) return fail(h, EAD_ERR_STATE, "nothing to fetch: call ead_begin first");
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    const int cap = h->s.cap;
    std::vector<int> ngen(h->batch);
    HIP_TRY(h, hipMemcpy(ngen.data(), h->s.ngen, h->batch * sizeof(int), hipMemcpyDeviceToHost));
    for (int b = 0; b < h->batch; ++b) {
        const int n = ngen[b];
        if (n > stride) return fail(h, EAD_ERR_INVALID_ARG, "stride %d smaller than %d generated tokens", stride, n);
        if (lens) lens[b] = n;
        if (!n) continue;
        if (tok) HIP_TRY(h, hipMemcpy(tok + (size_t)b * stride, h->s.out_tok + (size_t)b * cap, n * sizeof(int), hipMemcpyDeviceToHost));
        if (mid) HIP_TRY(h, hipMemcpy(mid + (size_t)b * stride, h->s.out_mid + (size_t)b * cap, n, hipMemcpyDeviceToHost));
        if (H) HIP_TRY(h, hipMemcpy(H + (size_t)b * stride, h->s.out_H + (size_t)b * cap, n * sizeof(float), hipMemcpyDeviceToHost));
        if (Hbar) HIP_TRY(h, hipMemcpy(Hbar + (size_t)b * stride, h->s.out_Hbar + (size_t)b * cap, n * sizeof(float), hipMemcpyDeviceToHost));
        if (dec) HIP_TRY(h, hipMemcpy(dec + (size_t)b * stride, h->s.out_dec + (size_t)b * cap, n, hipMemcpyDeviceToHost));
    }
    return EAD_OK;
}

// ---- stand-alone entropy: where the partials of a pass go ----------------------------------
// ead_entropy_argmax: a per-device buffer that the first call on a device allocates (kept until the
// process ends).  A gate owns a buffer of its own.  ead_entropy_argmax_static: the file-scope device
// array below, for callers that must not allocate.
constexpr int kEntMaxRows = 4096, kEntMaxChunks = 64;
constexpr int kEntStaticPartials = 16384;              // rows * chunks a call of ead_entropy_argmax_static may need
constexpr int kEntMaxDevices = 16;

static __device__ __align__(256) unsigned char scratch[(size_t)kEntStaticPartials * sizeof(EntPartial)];

struct EntDevice {                // per device, set up once by the first call on it
    bool ready = false;
    int resident = 1024;          // workgroups of k_entropy_partial the chip holds at once
    EntPartial *static_part = nullptr;     // device address of `scratch` on this device
    EntPartial *heap_part = nullptr;       // ead_entropy_argmax's buffer, allocated on first use
};
EntDevice g_ent_dev[kEntMaxDevices];
std::mutex g_ent_mutex;

// Device record of the current device; allocates nothing.
ead_status entropy_device(EntDevice **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(nullptr, EAD_ERR_NO_DEVICE, "no HIP device");
    if (dev < 0 || dev >= kEntMaxDevices) return fail(nullptr, EAD_ERR_DEVICE, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_ent_mutex);
    EntDevice &d = g_ent_dev[dev];
    if (!d.ready) {
        // every GPU holds its own copy of the array at its own address: ask with this device current
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(nullptr, EAD_ERR_DEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        d.static_part = (EntPartial *)p;
        int per_cu = 0;
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_entropy_partial<bf16_t>, 256, 0) == hipSuccess && per_cu > 0)
            d.resident = per_cu * prop.multiProcessorCount;
        d.ready = true;
    }
    *out = &d;
    return EAD_OK;
}

ead_status entropy_heap_scratch(EntDevice *d, EntPartial **out) {
    std::lock_guard<std::mutex> lock(g_ent_mutex);
    if (!d->heap_part) {
        void *p = nullptr;
        if (hipMalloc(&p, sizeof(EntPartial) * (size_t)kEntMaxRows * kEntMaxChunks) != hipSuccess)
            return fail(nullptr, EAD_ERR_OOM, "scratch allocation failed");
        d->heap_part = (EntPartial *)p;
    }
    *out = d->heap_part;
    return EAD_OK;
}

// The split of a row into work items depends on (rows, V) alone, so a step's result does not depend on
// how many steps share a launch, nor on which entry point asked for it.  Long chunks (up to 8 vectors
// per thread) amortise the per-workgroup merge; shorter ones only when the rows of one step would
// otherwise give too few workgroups to fill the chip.
void entropy_split(int rows, int V, int *chunks_out, int *per_out) {
    const int nvec = V / 8;
    int chunks = std::max(1, (nvec + 2047) / 2048);
    while ((long)chunks * rows < 512 && chunks < kEntMaxChunks && nvec / (chunks * 2) >= 256) chunks *= 2;
    int per = (std::max(nvec, 1) + chunks - 1) / chunks;
    while (per > 8 * 256) { ++chunks; per = (nvec + chunks - 1) / chunks; }
    *chunks_out = chunks; *per_out = per;
}

template <typename T>
void launch_entropy_partial(const void *const *step_logits, int steps, int rows, int V, EntPartial *part, int resident,
                            hipStream_t st) {
    int chunks, per;
    entropy_split(rows, V, &chunks, &per);
    EntArgs<T> a{};
    for (int z = 0; z < steps; ++z) a.step_logits[z] = (const T *)step_logits[z];
    a.V = V; a.rows = rows; a.chunks = chunks; a.vec_per_item = per; a.items = steps * rows * chunks; a.partials = part;
    // persistent grid: as many workgroups as the chip holds at once
    hipLaunchKernelGGL((k_entropy_partial<T>), dim3(std::min(a.items, resident)), dim3(256), 0, st, a);
}

ead_status entropy_check(const void *const *step_logits, int steps, int dtype, int rows, int vocab) {
    if (steps < 1 || steps > kGateMaxSteps || (long)steps * rows > kEntMaxRows)
        return fail(nullptr, EAD_ERR_INVALID_ARG, "too many steps for one launch");
    for (int z = 0; z < steps; ++z)
        if (!step_logits[z]) return fail(nullptr, EAD_ERR_INVALID_ARG, "null logits pointer");
    if (rows < 1 || rows > kEntMaxRows) return fail(nullptr, EAD_ERR_INVALID_ARG, "rows must be in 1..%d", kEntMaxRows);
    if (vocab < 1) return fail(nullptr, EAD_ERR_INVALID_ARG, "vocab must be >= 1");
    if (dtype != EAD_F32 && dtype != EAD_BF16) return fail(nullptr, EAD_ERR_INVALID_ARG, "unknown dtype");
    if (vocab % 8) return fail(nullptr, EAD_ERR_SHAPE, "vocab must be a multiple of 8");
    if ((long)vocab > 64L * 2048 * 8) return fail(nullptr, EAD_ERR_SHAPE, "vocab above %ld", 64L * 2048 * 8);
    return EAD_OK;
}

// step_logits: host array of `steps` device pointers (<= kGateMaxSteps), one [rows, vocab] matrix each;
// part: room for steps * rows * chunks partials (chunks as entropy_split gives it)
void entropy_launch(const void *const *step_logits, int steps, int dtype, int rows, int vocab, hipStream_t st,
                    EntPartial *part, int resident) {
    if (dtype == EAD_BF16) launch_entropy_partial<bf16_t>(step_logits, steps, rows, vocab, part, resident, st);
    else launch_entropy_partial<float>(step_logits, steps, rows, vocab, part, resident, st);
}

template <typename T>
void launch_entropy_rows(const void *const *step_logits, int steps, int rows, int V, int resident, hipStream_t st,
                         const GateStepArgs &gate, float *pair_H, int *row_tickets) {
    const int nvec = V / 8;
    EntRowArgs<T> a{};
    for (int z = 0; z < steps; ++z) a.step_logits[z] = (const T *)step_logits[z];
    a.V = V; a.rows = rows; a.steps = steps;
    a.chunks = std::max(1, (nvec + 2047) / 2048);                 // pieces of at most 8 vectors per thread
    a.vec_per_item = (std::max(nvec, 1) + a.chunks - 1) / a.chunks;
    a.pair_H = pair_H; a.row_tickets = row_tickets; a.gate = gate;
    hipLaunchKernelGGL((k_entropy_rows<T>), dim3(std::min(steps * rows, resident)), dim3(256), 0, st, a);
}

}  // namespace

struct ead_gate {
    GateState st; GateCfg cfg; int rows; hipStream_t stream;
    EntPartial *part = nullptr;   // partials of this gate's entropy passes: (steps per launch) x rows x kEntMaxChunks
    float *pair_H = nullptr;      // small windows (one launch per group of steps): entropies handed between workgroups
    int *row_tickets = nullptr;   //   and the arrival counters per row, zero between launches
    int resident = 1024;
    std::vector<void *> allocs;
};

// ======================================================================================
// C ABI
// ======================================================================================
extern "C" {

int32_t ead_version(void) { return 100; }

const char *ead_last_error(const ead_handle *h) { return h ? h->err.c_str() : g_create_error.c_str(); }

void ead_destroy(ead_handle *h) {
    if (!h) return;
    (void)hipStreamSynchronize(h->lanes[0].stream);
    if (h->lane1_stream) { (void)hipStreamSynchronize(h->lane1_stream); (void)hipStreamDestroy(h->lane1_stream); }
    for (auto &l : h->lanes) {
        if (l.rb_model) (void)hipHostFree(l.rb_model);
        if (l.rb_done) (void)hipHostFree(l.rb_done);
        if (l.done_ev) (void)hipEventDestroy(l.done_ev);
    }
    for (void *p : h->allocs) (void)hipFree(p);
    if (h->h_model) (void)hipHostFree(h->h_model);
    if (h->h_done) (void)hipHostFree(h->h_done);
    prof_collect(h);
    for (hipEvent_t e : h->ev_pool) (void)hipEventDestroy(e);
    delete h;
}

ead_status ead_create(const ead_model_desc *small_model, const ead_model_desc *large_model, const ead_params *p,
                      ead_handle **out) {
    if (!out) return fail(nullptr, EAD_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!p) return fail(nullptr, EAD_ERR_INVALID_ARG, "params is null");
    TRY(check_model(small_model, "small"));
    TRY(check_model(large_model, "large"));
    if (small_model->vocab != large_model->vocab)
        return fail(nullptr, EAD_ERR_VOCAB_MISMATCH, "vocab sizes differ: %d vs %d", small_model->vocab, large_model->vocab);
    if (p->window < 1 || p->d_min < 1 || !(p->tau == p->tau) || p->max_batch < 1 || p->max_seq < 2 ||
        (p->unit != EAD_NATS && p->unit != EAD_BITS))
        return fail(nullptr, EAD_ERR_INVALID_ARG, "need window >= 1, d_min >= 1, tau not NaN, max_batch >= 1, max_seq >= 2, unit 0/1");
    if (p->window > 4096) return fail(nullptr, EAD_ERR_INVALID_ARG, "window above 4096");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(nullptr, EAD_ERR_NO_DEVICE, "no HIP device available");

    ead_handle *h = new (std::nothrow) ead_handle();
    if (!h) return fail(nullptr, EAD_ERR_OOM, "host allocation failed");
    h->prm = *p; h->stream = (hipStream_t)p->hip_stream; h->force_model = -1;
    h->cfg = GateCfg{p->window, p->tau, p->d_min};
    ead_status rc = EAD_OK;
    auto body = [&]() -> ead_status {
        // internal strides are rounded up to whole 32-key blocks (the matrix-core attention reads such
        // blocks of the transposed V copy); the caller's limit stays p->max_seq
        const int MB = p->max_batch, MS = (p->max_seq + 31) & ~31;
        TRY(small_model->dtype == EAD_BF16 ? build_model<bf16_t>(h, small_model, &h->mdl[0], MB, MS)
                                           : build_model<float>(h, small_model, &h->mdl[0], MB, MS));
        TRY(large_model->dtype == EAD_BF16 ? build_model<bf16_t>(h, large_model, &h->mdl[1], MB, MS)
                                           : build_model<float>(h, large_model, &h->mdl[1], MB, MS));
        const long total = (long)MB * MS;
        h->Tmax = (int)std::min<long>(std::max<long>(MB, 1024), std::max<long>(total, MB));
        h->Tmax = (h->Tmax + 15) & ~15;
        h->items_max = std::max(h->Tmax, 2048);
        h->lm_grid = 1024;
        h->score_rows = 160;         // rows per teacher-forced pass (two 128-row sweeps at most)
        SeqState &s = h->s;
        s.max_batch = MB; s.max_seq = MS; s.cap = MS;
        TRY(dmalloc(h, &s.tokens, (size_t)MB * MS)); TRY(dmalloc(h, &s.len, (size_t)MB)); TRY(dmalloc(h, &s.kvlen, (size_t)2 * MB));
        TRY(dmalloc(h, &s.model, (size_t)MB)); TRY(dmalloc(h, &s.c, (size_t)MB)); TRY(dmalloc(h, &s.ngen, (size_t)MB));
        TRY(dmalloc(h, &s.done, (size_t)MB)); TRY(dmalloc(h, &s.last_step, (size_t)MB)); TRY(dmalloc(h, &s.goal, (size_t)MB));
        TRY(dmalloc(h, &s.ring, (size_t)MB * 4096)); TRY(dmalloc(h, &s.err, (size_t)1));
        TRY(dmalloc(h, &s.out_tok, (size_t)MB * MS)); TRY(dmalloc(h, &s.out_mid, (size_t)MB * MS));
        TRY(dmalloc(h, &s.out_H, (size_t)MB * MS)); TRY(dmalloc(h, &s.out_Hbar, (size_t)MB * MS));
        TRY(dmalloc(h, &s.out_dec, (size_t)MB * MS));
        TRY(dmalloc(h, &s.forced_tok, (size_t)MB * MS)); TRY(dmalloc(h, &s.forced_mid, (size_t)MB * MS));
        const Model &a = h->mdl[0], &b = h->mdl[1];
        const size_t dmax = std::max(a.d, b.d), qmax = std::max(a.H * a.hd, b.H * b.hd), fmax_ = std::max(a.F, b.F);
        const size_t T = h->Tmax;
        // per-lane scratch: allocated twice when two passes may run side by side
        auto alloc_lane = [&]() -> ead_status {
            TRY(dmalloc(h, &h->plan.hdr, (size_t)4)); TRY(dmalloc(h, &h->plan.row_seq, (size_t)h->Tmax));
            TRY(dmalloc(h, &h->plan.row_pos, (size_t)h->Tmax));
            TRY(dmalloc(h, &h->plan.lm_row, (size_t)h->Tmax)); TRY(dmalloc(h, &h->plan.lm_seq, (size_t)h->Tmax));
            TRY(dmalloc(h, &h->x, T * dmax)); TRY(dmalloc(h, &h->q, T * qmax)); TRY(dmalloc(h, &h->o, T * qmax));
            TRY(dmalloc(h, &h->hbuf, T * fmax_));
            TRY(dmalloc(h, &h->xp_a, T * dmax)); TRY(dmalloc(h, &h->xp_o, T * qmax)); TRY(dmalloc(h, &h->xp_h, T * fmax_));
            HIP_TRY(h, hipMemsetAsync(h->xp_a, 0, T * dmax * 2, h->stream));
            HIP_TRY(h, hipMemsetAsync(h->xp_o, 0, T * qmax * 2, h->stream));
            HIP_TRY(h, hipMemsetAsync(h->xp_h, 0, T * fmax_ * 2, h->stream));
            TRY(dmalloc(h, &h->part_o, (size_t)h->items_max * qmax)); TRY(dmalloc(h, &h->part_ml, (size_t)h->items_max * std::max(a.H, b.H)));
            TRY(dmalloc(h, &h->tickets, (size_t)h->Tmax * std::max(a.H, b.H)));
            TRY(dmalloc(h, &h->sk_part, kSplitKFloats)); TRY(dmalloc(h, &h->sk_tickets, (size_t)kSplitKGroups));
            HIP_TRY(h, hipMemsetAsync(h->sk_tickets, 0, kSplitKGroups * sizeof(int), h->stream));
            HIP_TRY(h, hipMemsetAsync(h->tickets, 0, (size_t)h->Tmax * std::max(a.H, b.H) * sizeof(int), h->stream));
            TRY(dmalloc(h, &h->lm_part, std::max((size_t)std::max<size_t>(MB, h->score_rows) * h->lm_grid, (size_t)256 * kFusedRbChunk)));
            return EAD_OK;
        };
        h->two_lanes = (MB > 1 && MB <= 64 * kAllowWords) ? 1 : 0;
        TRY(alloc_lane());
        save_lane(h, 0);
        h->lanes[0].stream = h->stream;
        if (h->two_lanes) {
            TRY(alloc_lane());
            save_lane(h, 1);
            HIP_TRY(h, hipStreamCreateWithFlags(&h->lane1_stream, hipStreamNonBlocking));   // default priority
            h->lanes[1].stream = h->lane1_stream;
        }
        for (int i = 0; i < (h->two_lanes ? 2 : 1); ++i) {
            HIP_TRY(h, hipHostMalloc((void **)&h->lanes[i].rb_model, std::max<size_t>(MB, 64) * sizeof(int), hipHostMallocDefault));
            HIP_TRY(h, hipHostMalloc((void **)&h->lanes[i].rb_done, std::max<size_t>(MB, 64) * sizeof(int), hipHostMallocDefault));
            HIP_TRY(h, hipEventCreateWithFlags(&h->lanes[i].done_ev, hipEventDisableTiming));
        }
        {
            const int keep = h->two_lanes;      // use_lane maps every lane to 0 when there is one
            h->two_lanes = 1; use_lane(h, 0); h->two_lanes = keep;
        }
        TRY(dmalloc(h, &h->logits_dump, (size_t)h->score_rows * a.V));
        TRY(dmalloc(h, &h->sc_H, (size_t)MS)); TRY(dmalloc(h, &h->sc_arg, (size_t)MS));
        {
            const size_t hmax = std::max(a.H, b.H), qm = qmax;
            TRY(dmalloc(h, &h->att_o, qm * kFusedMaxSplits)); TRY(dmalloc(h, &h->att_ml, hmax * kFusedMaxSplits));
            TRY(dmalloc(h, &h->bar_mem, (size_t)kBarGroups * 32 + 32)); TRY(dmalloc(h, &h->abort_flag, (size_t)1));
            HIP_TRY(h, hipMemsetAsync(h->bar_mem, 0, (kBarGroups * 32 + 32) * sizeof(unsigned), h->stream));
            HIP_TRY(h, hipMemsetAsync(h->abort_flag, 0, sizeof(int), h->stream));
            int dev = 0; hipDeviceProp_t prop;
            HIP_TRY(h, hipGetDevice(&dev)); HIP_TRY(h, hipGetDeviceProperties(&prop, dev));
            h->fused_grid = std::min(256, prop.multiProcessorCount);
            h->n_cu = prop.multiProcessorCount;
            h->lds_per_block = std::max<size_t>(prop.sharedMemPerBlock, prop.sharedMemPerBlockOptin);
            for (int mi = 0; mi < 2; ++mi) {
                Model &md = h->mdl[mi];
                void *fn = fused_kernel_for(md);
                int per_cu = 0;
                md.fused_ok = fn && prop.cooperativeLaunch && md.n_mats <= kFusedMaxMats &&
                              hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fused_lds_bytes(md)) == hipSuccess &&
                              hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kFusedThreads, fused_lds_bytes(md)) == hipSuccess &&
                              per_cu >= 1 && md.KV * kFusedMaxSplits <= h->fused_grid;
                void *sfn = stream_kernel_for(md);
                per_cu = 0;
                md.stream_ok = md.fused_ok && sfn && stream_lds_bytes(md) <= h->lds_per_block &&
                               hipFuncSetAttribute(sfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)stream_lds_bytes(md)) == hipSuccess &&
                               hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sfn, kStreamThreads, stream_lds_bytes(md)) == hipSuccess &&
                               per_cu >= 1;
            }
        }
        HIP_TRY(h, hipHostMalloc((void **)&h->h_model, std::max<size_t>((size_t)MB * MS, 64) * sizeof(int), hipHostMallocDefault));
        HIP_TRY(h, hipHostMalloc((void **)&h->h_done, std::max<size_t>(MB, 64) * sizeof(int), hipHostMallocDefault));
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        HIP_TRY(h, hipGetLastError());
        return EAD_OK;
    };
    rc = body();
    if (rc != EAD_OK) { g_create_error = h->err; ead_destroy(h); return rc; }
    *out = h;
    return EAD_OK;
}

ead_status ead_set_gate(ead_handle *h, int32_t window, float tau, int32_t d_min, int32_t unit, int32_t eos_id) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (window < 1 || window > 4096 || d_min < 1 || !(tau == tau) || (unit != EAD_NATS && unit != EAD_BITS))
        return fail(h, EAD_ERR_INVALID_ARG, "need 1 <= window <= 4096, d_min >= 1, tau not NaN, unit 0/1");
    h->prm.window = window; h->prm.tau = tau; h->prm.d_min = d_min; h->prm.unit = unit; h->prm.eos_id = eos_id;
    h->cfg = GateCfg{window, tau, d_min};
    h->began = 0;
    return EAD_OK;
}

ead_status ead_force_model(ead_handle *h, int32_t which) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (which < -1 || which > 1) return fail(h, EAD_ERR_INVALID_ARG, "model must be -1, 0 or 1");
    h->force_model = which; h->began = 0;
    return EAD_OK;
}

ead_status ead_begin(ead_handle *h, const int32_t *prompt_tokens, const int32_t *prompt_lens, int32_t batch,
                     int32_t max_new_tokens) {
    if (!h) return EAD_ERR_INVALID_ARG;
    h->replay = 0; h->n_new = 0;
    return begin_impl(h, prompt_tokens, prompt_lens, batch, max_new_tokens);
}

ead_status ead_rewind(ead_handle *h, int32_t max_new_tokens) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (!h->prefilled) return fail(h, EAD_ERR_STATE, "ead_rewind needs the prompts of a previous ead_begin in the caches");
    if (max_new_tokens < 1) return fail(h, EAD_ERR_INVALID_ARG, "max_new_tokens must be >= 1");
    for (int b = 0; b < h->batch; ++b)
        if ((long)h->prompt_len[b] + max_new_tokens > h->prm.max_seq)
            return fail(h, EAD_ERR_SEQ_OVERFLOW, "prompt %d: %d + %d tokens exceed max_seq %d", b, h->prompt_len[b], max_new_tokens, h->prm.max_seq);
    use_lane(h, 0);
    if (h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1].stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    h->replay = 0; h->n_new = 0;
    TRY(reset_run_state(h, max_new_tokens, 1));
    memset(&h->stats, 0, sizeof h->stats);
    h->began = 1;
    return EAD_OK;
}

ead_status ead_decode(ead_handle *h, int32_t n_steps) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (n_steps < 0) return fail(h, EAD_ERR_INVALID_ARG, "n_steps < 0");
    return decode_impl(h, n_steps);
}

ead_status ead_decode_tokens(ead_handle *h, int64_t n_tokens, int32_t max_lead) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (n_tokens < 0 || max_lead < 1) return fail(h, EAD_ERR_INVALID_ARG, "need n_tokens >= 0 and max_lead >= 1");
    if (h->prm.max_batch > 64 * kAllowWords) return fail(h, EAD_ERR_INVALID_ARG, "ead_decode_tokens serves batches of up to %d sequences", 64 * kAllowWords);
    if (h->replay) return fail(h, EAD_ERR_STATE, "ead_decode_tokens inside a replay");
    return decode_impl(h, 0, (long)n_tokens, max_lead);
}

ead_status ead_fetch(ead_handle *h, int32_t stride, int32_t *out_tokens, uint8_t *out_model_id, float *out_entropy,
                     float *out_window_mean, int32_t *out_lens) {
    if (!h) return EAD_ERR_INVALID_ARG;
    return fetch_impl(h, stride, out_tokens, out_model_id, out_entropy, out_window_mean, nullptr, out_lens);
}

ead_status ead_generate(ead_handle *h, const int32_t *prompt_tokens, const int32_t *prompt_lens, int32_t batch,
                        int32_t max_new_tokens, int32_t *out_tokens, uint8_t *out_model_id, float *out_entropy,
                        float *out_window_mean, int32_t *out_lens) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (!out_tokens || !out_model_id || !out_entropy || !out_lens) return fail(h, EAD_ERR_INVALID_ARG, "null output pointer");
    TRY(ead_begin(h, prompt_tokens, prompt_lens, batch, max_new_tokens));
    TRY(decode_impl(h, max_new_tokens));
    return fetch_impl(h, max_new_tokens, out_tokens, out_model_id, out_entropy, out_window_mean, nullptr, out_lens);
}

ead_status ead_replay(ead_handle *h, const int32_t *prompt_tokens, const int32_t *prompt_lens, int32_t batch,
                      int32_t n_new, const int32_t *forced_tokens, const uint8_t *forced_model_id, int32_t *out_argmax,
                      float *out_entropy, float *out_window_mean, uint8_t *out_decision) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (!forced_tokens || !forced_model_id) return fail(h, EAD_ERR_INVALID_ARG, "null forced trajectory");
    TRY(validate_prompts(h, prompt_tokens, prompt_lens, batch, n_new));
    for (size_t i = 0; i < (size_t)batch * n_new; ++i) {
        if (forced_model_id[i] > 1) return fail(h, EAD_ERR_INVALID_ARG, "forced_model_id must be 0 or 1");
        if (forced_tokens[i] < 0 || forced_tokens[i] >= h->mdl[0].V) return fail(h, EAD_ERR_INVALID_ARG, "forced token out of range");
    }
    const int cap = h->s.cap;
    // stage the forced trajectory with the device row stride; keep the ids on the host too
    std::vector<int> ft((size_t)batch * cap, 0); std::vector<uint8_t> fm((size_t)batch * cap, 0);
    for (int b = 0; b < batch; ++b)
        for (int i = 0; i < n_new; ++i) {
            ft[(size_t)b * cap + i] = forced_tokens[(size_t)b * n_new + i];
            fm[(size_t)b * cap + i] = forced_model_id[(size_t)b * n_new + i];
            h->h_model[(size_t)b * cap + i] = forced_model_id[(size_t)b * n_new + i];
        }
    HIP_TRY(h, hipMemcpyAsync(h->s.forced_tok, ft.data(), ft.size() * sizeof(int), hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipMemcpyAsync(h->s.forced_mid, fm.data(), fm.size(), hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    const int saved_force = h->force_model;
    h->force_model = -1; h->replay = 1; h->n_new = n_new;
    ead_status rc = begin_impl(h, prompt_tokens, prompt_lens, batch, n_new);
    if (rc == EAD_OK) {
        // the first token's model is dictated as well
        std::vector<int> model(h->s.max_batch, 0);
        for (int b = 0; b < batch; ++b) { h->hs[b].model = forced_model_id[(size_t)b * n_new]; model[b] = h->hs[b].model; }
        hipError_t e = hipMemcpy(h->s.model, model.data(), model.size() * sizeof(int), hipMemcpyHostToDevice);
        if (e != hipSuccess) rc = fail(h, EAD_ERR_DEVICE, "hipMemcpy: %s", hipGetErrorString(e));
    }
    if (rc == EAD_OK) rc = decode_impl(h, n_new);
    if (rc == EAD_OK) rc = fetch_impl(h, n_new, out_argmax, nullptr, out_entropy, out_window_mean, out_decision, nullptr);
    h->replay = 0; h->force_model = saved_force; h->began = 0; h->prefilled = 0;
    return rc;
}

ead_status ead_score(ead_handle *h, int32_t which, const int32_t *tokens, int32_t len, float *out_logits,
                     float *out_entropy, int32_t *out_argmax) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (which != 0 && which != 1) return fail(h, EAD_ERR_INVALID_ARG, "model must be 0 or 1");
    if (!tokens || len < 1) return fail(h, EAD_ERR_INVALID_ARG, "need tokens and len >= 1");
    if (len > h->prm.max_seq) return fail(h, EAD_ERR_SEQ_OVERFLOW, "len %d exceeds max_seq %d", len, h->prm.max_seq);
    Model &m = h->mdl[which];
    for (int i = 0; i < len; ++i)
        if (tokens[i] < 0 || tokens[i] >= m.V) return fail(h, EAD_ERR_INVALID_ARG, "token %d out of range", i);
    use_lane(h, 0);
    hipStream_t st = h->stream;
    h->began = 0; h->batch = 1; h->replay = 0; h->prefilled = 0;
    struct Scoring { ead_handle *h; Scoring(ead_handle *h_) : h(h_) { h->scoring = 1; } ~Scoring() { h->scoring = 0; } } scoring_guard(h);
    h->hs.assign(1, HostSeq{});
    HostSeq &s = h->hs[0];
    s.len = len; s.model = which; s.last_step = -1; s.ngen = 0; s.goal = 1;
    const int zero = 0, one_len = len, neg = -1, one = 1;
    HIP_TRY(h, hipMemcpyAsync(h->s.tokens, tokens, len * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.len, &one_len, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.kvlen + which * h->s.max_batch, &zero, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.model, &which, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.done, &zero, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.last_step, &neg, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.ngen, &zero, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(h->s.goal, &one, sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipStreamSynchronize(st));
    std::vector<int> rows; std::vector<char> complete;
    for (;;) {
        int n_lm, ctx_max;
        const int first = s.kvlen[which];
        const int T = host_plan(h, which, h->score_rows, 0, 2, false, -1, &n_lm, &ctx_max, &rows, &complete);
        if (T == 0) break;
        launch_plan(h, which, h->score_rows, 0, 2, false, -1);
        TRY(run_pass(h, which, T, n_lm, ctx_max, out_logits != nullptr, rows));
        launch_finalize(h, which, n_lm, true);
        s.kvlen[which] += T;
        if (out_logits) {
            HIP_TRY(h, hipMemcpyAsync(out_logits + (size_t)first * m.V, h->logits_dump, (size_t)T * m.V * sizeof(float),
                                      hipMemcpyDeviceToHost, st));
            HIP_TRY(h, hipStreamSynchronize(st));
        }
    }
    HIP_TRY(h, hipStreamSynchronize(st));
    if (out_entropy) HIP_TRY(h, hipMemcpy(out_entropy, h->sc_H, len * sizeof(float), hipMemcpyDeviceToHost));
    if (out_argmax) HIP_TRY(h, hipMemcpy(out_argmax, h->sc_arg, len * sizeof(int), hipMemcpyDeviceToHost));
    return EAD_OK;
}

ead_status ead_get_stats(ead_handle *h, ead_stats *out) {
    if (!h || !out) return EAD_ERR_INVALID_ARG;
    *out = h->stats;
    const double n = (double)(h->stats.tokens_small + h->stats.tokens_large);
    out->large_share = n > 0 ? h->stats.tokens_large / n : 0.0;
    out->param_ratio = ((1.0 - out->large_share) * h->mdl[0].n_params + out->large_share * h->mdl[1].n_params) / h->mdl[1].n_params;
    return EAD_OK;
}

ead_status ead_reset_stats(ead_handle *h) {
    if (!h) return EAD_ERR_INVALID_ARG;
    memset(&h->stats, 0, sizeof h->stats);
    return EAD_OK;
}

ead_status ead_set_schedule(ead_handle *h, int32_t grouped, float start_fraction, float stop_fraction) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (grouped && !(start_fraction > 0.f && start_fraction <= 1.f && stop_fraction >= 0.f && stop_fraction <= start_fraction))
        return fail(h, EAD_ERR_INVALID_ARG, "need 0 < start_fraction <= 1 and 0 <= stop_fraction <= start_fraction");
    h->sched_grouped = grouped ? 1 : 0; h->sched_phase = 0;
    if (grouped) { h->sched_hi = start_fraction; h->sched_lo = stop_fraction; }
    return EAD_OK;
}

ead_status ead_set_sampling(ead_handle *h, float temperature, uint64_t seed) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (!(temperature >= 0.f) || !std::isfinite(temperature)) return fail(h, EAD_ERR_INVALID_ARG, "temperature must be finite and >= 0");
    h->samp_temp = temperature; h->samp_seed = seed;
    return EAD_OK;
}

ead_status ead_set_fused(ead_handle *h, int32_t on) {
    if (!h) return EAD_ERR_INVALID_ARG;
    h->fused_on = on == 2 ? 2 : (on ? 1 : 0);     // 2: the register-buffered kernel even where the streamed one is available
    return EAD_OK;
}

ead_status ead_profile_enable(ead_handle *h, int32_t on) {
    if (!h) return EAD_ERR_INVALID_ARG;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    if (h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1].stream));
    prof_collect(h);
    memset(h->prof_ms, 0, sizeof h->prof_ms); memset(h->prof_bytes, 0, sizeof h->prof_bytes); memset(h->prof_n, 0, sizeof h->prof_n);
    h->prof_on = on ? 1 : 0;
    return EAD_OK;
}

ead_status ead_profile_select(ead_handle *h, const char *name) {
    if (!h) return EAD_ERR_INVALID_ARG;
    if (!name || !*name) { h->prof_mask = ~0ull; return EAD_OK; }
    unsigned long long mask = 0;
    for (int c = 0; c < PK_COUNT * 2; ++c) {
        char buf[64];
        snprintf(buf, sizeof buf, "%s/%s", kProfNames[c / 2], (c & 1) ? "large" : "small");
        if (strcmp(buf, name) == 0) mask |= 1ull << c;
    }
    if (!mask) return fail(h, EAD_ERR_INVALID_ARG, "no kernel class is called '%s'", name);
    h->prof_mask = mask;
    return EAD_OK;
}

ead_status ead_profile_read(ead_handle *h, ead_kernel_profile *out, int32_t capacity, int32_t *n_out) {
    if (!h || !out || !n_out || capacity < 0) return EAD_ERR_INVALID_ARG;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    if (h->two_lanes) HIP_TRY(h, hipStreamSynchronize(h->lanes[1].stream));
    prof_collect(h);
    int n = 0;
    for (int c = 0; c < PK_COUNT * 2 && n < capacity; ++c) {
        if (!h->prof_n[c]) continue;
        snprintf(out[n].name, sizeof out[n].name, "%s/%s", kProfNames[c / 2], (c & 1) ? "large" : "small");
        out[n].launches = h->prof_n[c]; out[n].total_ms = h->prof_ms[c]; out[n].bytes = h->prof_bytes[c];
        ++n;
    }
    *n_out = n;
    return EAD_OK;
}

// ---- entropy / gate on their own ---------------------------------------------------------
namespace {
ead_status entropy_argmax_impl(const void *logits_dev, int32_t dtype, int32_t rows, int32_t vocab, int32_t unit,
                               float *H_dev, int32_t *argmax_dev, hipStream_t st, bool use_static) {
    if (!H_dev) return fail(nullptr, EAD_ERR_INVALID_ARG, "H_dev is null");
    if (unit != EAD_NATS && unit != EAD_BITS) return fail(nullptr, EAD_ERR_INVALID_ARG, "unit must be 0 or 1");
    TRY(entropy_check(&logits_dev, 1, dtype, rows, vocab));
    int chunks = 0, per = 0;
    entropy_split(rows, vocab, &chunks, &per);
    EntDevice *d = nullptr;
    TRY(entropy_device(&d));
    EntPartial *part = nullptr;
    if (use_static) {
        if ((long)rows * chunks > kEntStaticPartials)
            return fail(nullptr, EAD_ERR_INVALID_ARG, "rows * chunks = %d * %d exceeds the %d partials of the static scratch array",
                        rows, chunks, kEntStaticPartials);
        part = d->static_part;
    } else {
        TRY(entropy_heap_scratch(d, &part));
    }
    entropy_launch(&logits_dev, 1, dtype, rows, vocab, st, part, d->resident);
    hipLaunchKernelGGL(k_entropy_finalize, dim3(rows), dim3(64), 0, st, part, chunks, rows, unit, H_dev, argmax_dev);
    if (hipGetLastError() != hipSuccess) return fail(nullptr, EAD_ERR_DEVICE, "kernel launch failed");
    return EAD_OK;
}
}  // namespace

ead_status ead_entropy_argmax(const void *logits_dev, int32_t dtype, int32_t rows, int32_t vocab, int32_t unit,
                              float *H_dev, int32_t *argmax_dev, void *hip_stream) {
    return entropy_argmax_impl(logits_dev, dtype, rows, vocab, unit, H_dev, argmax_dev, (hipStream_t)hip_stream, false);
}

ead_status ead_entropy_argmax_static(const void *logits_dev, int32_t dtype, int32_t rows, int32_t vocab, int32_t unit,
                                     float *H_dev, int32_t *argmax_dev, void *hip_stream) {
    return entropy_argmax_impl(logits_dev, dtype, rows, vocab, unit, H_dev, argmax_dev, (hipStream_t)hip_stream, true);
}

ead_status ead_gate_create(int32_t rows, int32_t window, float tau, int32_t d_min, void *hip_stream, ead_gate **out) {
    if (!out) return fail(nullptr, EAD_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (rows < 1 || rows > kEntMaxRows || window < 1 || window > 4096 || d_min < 1 || !(tau == tau))
        return fail(nullptr, EAD_ERR_INVALID_ARG, "need 1 <= rows <= %d, 1 <= window <= 4096, d_min >= 1, tau not NaN", kEntMaxRows);
    ead_gate *g = new (std::nothrow) ead_gate();
    if (!g) return fail(nullptr, EAD_ERR_OOM, "host allocation failed");
    g->rows = rows; g->cfg = GateCfg{window, tau, d_min}; g->stream = (hipStream_t)hip_stream;
    EntDevice *d = nullptr;
    { const ead_status rc = entropy_device(&d); if (rc != EAD_OK) { delete g; return rc; } }
    g->resident = d->resident;
    const size_t steps_per_launch = std::max(1, std::min(kGateMaxSteps, kEntMaxRows / rows));
    void *p[7] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    const size_t sz[7] = {(size_t)rows * window * 4, (size_t)rows * 4, (size_t)rows * 4, (size_t)rows * 4,
                          steps_per_launch * rows * kEntMaxChunks * sizeof(EntPartial), steps_per_launch * rows * 4, (size_t)rows * 4};
    for (int i = 0; i < 7; ++i) {
        if (hipMalloc(&p[i], sz[i]) != hipSuccess) { for (int j = 0; j < i; ++j) (void)hipFree(p[j]); delete g; return fail(nullptr, EAD_ERR_OOM, "hipMalloc failed"); }
        g->allocs.push_back(p[i]);
    }
    g->st.ring = (float *)p[0]; g->st.n = (int *)p[1]; g->st.c = (int *)p[2]; g->st.model = (int *)p[3];
    g->part = (EntPartial *)p[4]; g->pair_H = (float *)p[5]; g->row_tickets = (int *)p[6];
    *out = g;
    return ead_gate_reset(g);
}

ead_status ead_gate_reset(ead_gate *g) {
    if (!g) return EAD_ERR_INVALID_ARG;
    (void)hipMemsetAsync(g->st.ring, 0, (size_t)g->rows * g->cfg.w * 4, g->stream);
    (void)hipMemsetAsync(g->st.n, 0, (size_t)g->rows * 4, g->stream);
    (void)hipMemsetAsync(g->st.c, 0, (size_t)g->rows * 4, g->stream);
    (void)hipMemsetAsync(g->st.model, 0, (size_t)g->rows * 4, g->stream);
    (void)hipMemsetAsync(g->row_tickets, 0, (size_t)g->rows * 4, g->stream);
    return hipGetLastError() == hipSuccess ? EAD_OK : EAD_ERR_DEVICE;
}

void ead_gate_destroy(ead_gate *g) {
    if (!g) return;
    (void)hipStreamSynchronize(g->stream);
    for (void *p : g->allocs) (void)hipFree(p);
    delete g;
}

ead_status ead_gate_step(ead_gate *g, const float *H_dev, uint8_t *model_id_dev, float *window_mean_dev,
                         uint8_t *next_model_dev) {
    if (!g || !H_dev) return EAD_ERR_INVALID_ARG;
    GateStepArgs a{};
    a.st = g->st; a.cfg = g->cfg; a.rows = g->rows; a.steps = 1; a.H = H_dev;
    a.model_id_out = model_id_dev; a.Hbar_out = window_mean_dev; a.next_out = next_model_dev;
    hipLaunchKernelGGL(k_gate_step, dim3(g->rows), dim3(64), 0, g->stream, a);
    return hipGetLastError() == hipSuccess ? EAD_OK : EAD_ERR_DEVICE;
}

namespace {
// Entropy + arg max of `ns` logits matrices and the gate through those steps.  Windows up to kGateFoldWindow: one
// launch (k_entropy_rows); longer windows: the partials pass, then k_gate_step.
ead_status gate_steps(ead_gate *g, const void *const *ptrs, int ns, int dtype, int vocab, int unit, float *H_dev,
                      int32_t *argmax_dev, uint8_t *model_id_dev, float *window_mean_dev, uint8_t *next_model_dev) {
    TRY(entropy_check(ptrs, ns, dtype, g->rows, vocab));
    GateStepArgs a{};
    a.st = g->st; a.cfg = g->cfg; a.rows = g->rows; a.steps = ns; a.unit = unit;
    a.H_out = H_dev; a.argmax_out = argmax_dev;
    a.model_id_out = model_id_dev; a.Hbar_out = window_mean_dev; a.next_out = next_model_dev;
    if (g->cfg.w <= kGateFoldWindow) {
        if (dtype == EAD_BF16) launch_entropy_rows<bf16_t>(ptrs, ns, g->rows, vocab, g->resident, g->stream, a, g->pair_H, g->row_tickets);
        else launch_entropy_rows<float>(ptrs, ns, g->rows, vocab, g->resident, g->stream, a, g->pair_H, g->row_tickets);
    } else {
        int chunks = 0, per = 0;
        entropy_split(g->rows, vocab, &chunks, &per);
        a.partials = g->part; a.n_part = chunks;
        entropy_launch(ptrs, ns, dtype, g->rows, vocab, g->stream, g->part, g->resident);
        hipLaunchKernelGGL(k_gate_step, dim3(g->rows), dim3(ns * 64), 0, g->stream, a);
    }
    return EAD_OK;
}
}  // namespace

ead_status ead_gate_step_logits(ead_gate *g, const void *logits_dev, int32_t dtype, int32_t vocab, int32_t unit,
                                float *H_dev, int32_t *argmax_dev, uint8_t *model_id_dev, float *window_mean_dev,
                                uint8_t *next_model_dev) {
    if (!g) return EAD_ERR_INVALID_ARG;
    if (unit != EAD_NATS && unit != EAD_BITS) return fail(nullptr, EAD_ERR_INVALID_ARG, "unit must be 0 or 1");
    TRY(gate_steps(g, &logits_dev, 1, dtype, vocab, unit, H_dev, argmax_dev, model_id_dev, window_mean_dev, next_model_dev));
    return hipGetLastError() == hipSuccess ? EAD_OK : EAD_ERR_DEVICE;
}

ead_status ead_gate_run_logits(ead_gate *g, const void *const *logits_dev_list, int32_t n_tensors, int32_t n_steps,
                               int32_t dtype, int32_t vocab, int32_t unit, float *H_dev, int32_t *argmax_dev,
                               uint8_t *model_id_dev, float *window_mean_dev) {
    if (!g || !logits_dev_list) return EAD_ERR_INVALID_ARG;
    if (n_tensors < 1 || n_tensors > 4096 || n_steps < 0) return fail(nullptr, EAD_ERR_INVALID_ARG, "need 1 <= n_tensors <= 4096, n_steps >= 0");
    if (unit != EAD_NATS && unit != EAD_BITS) return fail(nullptr, EAD_ERR_INVALID_ARG, "unit must be 0 or 1");
    for (int i = 0; i < n_tensors; ++i) if (!logits_dev_list[i]) return fail(nullptr, EAD_ERR_INVALID_ARG, "null logits pointer");
    // steps per launch, bounded by the gate's hand-over buffers
    const int S = std::max(1, std::min(kGateMaxSteps, kEntMaxRows / g->rows));
    for (int s0 = 0; s0 < n_steps; s0 += S) {
        const int ns = std::min(S, n_steps - s0);
        const void *ptrs[kGateMaxSteps];
        for (int z = 0; z < ns; ++z) ptrs[z] = logits_dev_list[(s0 + z) % n_tensors];
        const size_t o = (size_t)s0 * g->rows;
        TRY(gate_steps(g, ptrs, ns, dtype, vocab, unit, H_dev ? H_dev + o : nullptr, argmax_dev ? argmax_dev + o : nullptr,
                       model_id_dev ? model_id_dev + o : nullptr, window_mean_dev ? window_mean_dev + o : nullptr, nullptr));
    }
    return hipGetLastError() == hipSuccess ? EAD_OK : EAD_ERR_DEVICE;
}

}  // extern "C"
