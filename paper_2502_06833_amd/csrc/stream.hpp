// One decode step of one model for a single token row as ONE persistent kernel whose weight
// stream never stops: the bf16 variant of the fused step for the large shapes.
//
// A workgroup is eight consuming waves and two fetching waves.  The fetching waves walk, in
// order, every weight tile their workgroup will need during the whole step (all layers, then
// the LM head) and load it straight from global memory into a ring of 8 KB slots in LDS
// (global_load_lds, 16 bytes per lane); they hold no data in registers and never look at
// LDS, so nothing but the ring's capacity ever stops them.  While the consuming waves sit in a
// grid barrier, stage the next phase's activations or run the attention phase, the ring fills
// with the next matrix (about 4 us of stream at the chip's full rate), and the first row
// block of a phase is multiplied out of LDS the moment its activations are staged.
//
// A slot is 8 consecutive tiles of one 16-row block (one per consuming wave: wave w of slot t
// multiplies tile 8 t + w).  Hand-over is ONE hardware barrier per slot: the fetching waves
// arrive when slot i has landed, the consuming waves when they have read slot i - 1; behind it
// the consumers read slot i and the fetchers refill the ring position of slot i - 1.  The
// consuming waves also meet at the hardware barrier for their own reasons (staging, reductions,
// grid barriers); the fetching waves cannot look at LDS without stalling their loads (measured: a
// fetching wave that polls a counter in LDS between its loads streams at 3.8 instead of 6.3 TB/s over
// the chip), so they learn nothing from memory: they replay the fixed sequence of those meetings
// and arrive at each.  Should the consuming waves
// leave early (an abandoned grid barrier), the hardware barrier counts only the surviving waves
// and the fetching waves run their list to its end.
//
// Work split inside a phase is the same as in k_decode_fused: a workgroup owns 16-row blocks
// wg, wg+G, ... and its waves split K (interleaved by tile); partial sums meet in LDS and one
// wave, taking turns, finishes the row block after the next slot's barrier.
#pragma once
#include "fused.hpp"

namespace ead {

constexpr int kStreamDepth = 12;                 // ring slots
constexpr int kStreamSlotBytes = 8192;           // 8 tiles of 1 KB
constexpr int kStreamProducers = 2;
constexpr int kStreamLoads = kFusedWaves / kStreamProducers;   // tile loads per fetching wave and slot
constexpr int kStreamThreads = (kFusedWaves + kStreamProducers) * 64;
static_assert(kStreamLoads * (kStreamDepth - 1) <= 63, "outstanding loads must fit the vector memory counter");

// Where a model's packed weights are: matrix j (0 QKV, 1 output projection, 2 gate/up, 3 down)
// of layer l starts at base + l * layer_stride + off[j] (elements); index 4 is the LM head.
struct StreamModel {
    const bf16_t *base; size_t layer_stride; size_t off[4];
    const bf16_t *lm;
    int NB[5], KC[5];
    int L;
};

// Slots the workgroup `wg` of `G` takes during a step: both sides of the ring count the same.
__device__ __forceinline__ long stream_steps(const StreamModel &sm, int wg, int G) {
    long n = 0;
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        if (wg >= sm.NB[j]) continue;
        const long blocks = (sm.NB[j] - wg + G - 1) / G, nt = (sm.KC[j] + 7) >> 3;
        n += blocks * nt * (j < 4 ? sm.L : 1);
    }
    return n;
}

// The fetching waves' position in the list of slots of their workgroup: matrix (layer l, kind j),
// row block, slot.  Every member is the same in all lanes and lives in scalar registers: the
// description is copied out of the kernel arguments once, so that the loop around the loads
// touches no memory but the weights.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ size_t uni(size_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((size_t)hi << 32) | (size_t)lo;
}
struct StreamList {
    // the model
    size_t base, lm, stride, off0, off1, off2, off3;        // addresses in bytes
    int nb0, nb1, nb2, nb3, nb4, kc0, kc1, kc2, kc3, kc4, L, wg, G;
    // the position
    int l, j, rb, t, NB, KC, nt;
    size_t W;                                               // current matrix, byte address
    bool done;
    __device__ __forceinline__ explicit StreamList(const StreamModel &sm) {
        base = uni((size_t)sm.base); lm = uni((size_t)sm.lm); stride = uni(sm.layer_stride * sizeof(bf16_t));
        off0 = uni(sm.off[0] * sizeof(bf16_t)); off1 = uni(sm.off[1] * sizeof(bf16_t));
        off2 = uni(sm.off[2] * sizeof(bf16_t)); off3 = uni(sm.off[3] * sizeof(bf16_t));
        nb0 = uni(sm.NB[0]); nb1 = uni(sm.NB[1]); nb2 = uni(sm.NB[2]); nb3 = uni(sm.NB[3]); nb4 = uni(sm.NB[4]);
        kc0 = uni(sm.KC[0]); kc1 = uni(sm.KC[1]); kc2 = uni(sm.KC[2]); kc3 = uni(sm.KC[3]); kc4 = uni(sm.KC[4]);
        L = uni(sm.L); wg = uni((int)blockIdx.x); G = uni((int)gridDim.x);
        l = 0; j = 0; rb = 0; t = 0; NB = 0; KC = 1; nt = 1; W = 0; done = false;
    }
    __device__ __forceinline__ int nb_of(int jj) const { return jj == 0 ? nb0 : jj == 1 ? nb1 : jj == 2 ? nb2 : jj == 3 ? nb3 : nb4; }
    __device__ __forceinline__ int kc_of(int jj) const { return jj == 0 ? kc0 : jj == 1 ? kc1 : jj == 2 ? kc2 : jj == 3 ? kc3 : kc4; }
    // first matrix from (ll, jj) on in which this workgroup owns a row block; false if none is left
    __device__ __forceinline__ bool find(int &ll, int &jj) const {
        for (;;) {
            if (wg < nb_of(jj)) return true;
            if (jj == 4) return false;
            if (++jj == 4) { jj = 0; if (++ll == L) jj = 4; }
        }
    }
    __device__ __forceinline__ void enter(int ll, int jj) {
        l = ll; j = jj; NB = nb_of(jj); KC = kc_of(jj); nt = (KC + 7) >> 3; rb = wg; t = 0;
        const size_t off = jj == 0 ? off0 : jj == 1 ? off1 : jj == 2 ? off2 : off3;
        W = jj == 4 ? lm : base + (size_t)ll * stride + off;
    }
    __device__ __forceinline__ void open() { int ll = 0, jj = 0; if (find(ll, jj)) enter(ll, jj); else done = true; }
    // to the next slot; past the end of the list the position stays on the last slot
    __device__ __forceinline__ void next() {
        if (done) return;
        if (t + 1 < nt) { ++t; return; }
        if (rb + G < NB) { rb += G; t = 0; return; }
        if (j == 4) { done = true; return; }
        int ll = l, jj = j;
        if (++jj == 4) { jj = 0; if (++ll == L) jj = 4; }
        if (find(ll, jj)) enter(ll, jj); else done = true;
    }
};

typedef u32x4_t StreamRing[kFusedWaves][64];

// Request this fetching wave's tiles of the slot at the list position into `slot`, then move on.
// Tiles past the end of a row block re-read its last tile (they meet zeros in the multiply), so
// that every slot is the same number of loads and the wait counts stay fixed.
__device__ __forceinline__ void stream_issue(StreamList &pos, StreamRing &slot, int p, int lane) {
    const size_t row = pos.W + ((size_t)pos.rb * (size_t)pos.KC) * 1024 + (size_t)lane * 16;
#pragma unroll
    for (int q = 0; q < kStreamLoads; ++q) {
        const int tile = p + kStreamProducers * q;
        const int kc = min(pos.t * kFusedWaves + tile, pos.KC - 1);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + (size_t)kc * 1024),
                                         (__attribute__((address_space(3))) void *)&slot[tile][0], 16, 0, 0);
    }
    pos.next();
}

// ---- hardware barriers ---------------------------------------------------------------------------
// Every barrier of the workgroup is the hardware barrier and takes all ten waves.  The consuming
// waves meet at it for their own reasons too (staging, reductions, grid barriers): the number of
// such meetings per phase is fixed by the code below (kSync*), and the fetching waves, which have
// nothing to do there, simply arrive as many times (follow).
constexpr int kSyncGridBarrier = 2;      // bar_arrive + bar_wait
constexpr int kSyncStageNorm = 2;        // stage_norm_v / stage_norm_embed
constexpr int kSyncStageCopy = 1;        // stage_copy_v
constexpr int kSyncStageAttn = 1;        // stage_attn_v
constexpr int kSyncAttention = 1;        // fused_attention (or the lone barrier of a workgroup without a share)
constexpr int kSyncRowsEnd = 1;          // stream_rows, when the workgroup owned a row block

__device__ __forceinline__ void follow(int n) {
    for (int i = 0; i < n; ++i) asm volatile("s_barrier" ::: "memory");
}

// ---- device-coherent vector loads ---------------------------------------------------------------
// What other workgroups wrote during this kernel is read around the caches (see ld_coherent); these
// fetch 16 or 8 bytes per lane.  The loads are issued through asm, so the compiler does not know
// when their results arrive: the caller passes every result through coherent_wait before using it.
__device__ __forceinline__ f32x4e_t ld_coherent4_issue(const float *p) {
    f32x4e_t v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
typedef float f32x2e_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f32x2e_t ld_coherent2_issue(const float2 *p) {
    f32x2e_t v;
    asm volatile("global_load_dwordx2 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
template <int N>
__device__ __forceinline__ void coherent_wait(f32x4e_t (&v)[N]) {
    static_assert(N == 8, "one wait statement names all its registers");
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7])
                 :: "memory");
}

constexpr int kStageVecs = 8;            // 16-byte pieces per thread: K <= 8 * 4 * 512

// The staging routines run once per phase inside the kernel's long loop over phases, on the same
// buffers every time.  Passing a pointer through this keeps the per-thread addresses derived from it
// inside the phase (computed where they are used) instead of alive, in registers or spilled, across
// the whole loop.
template <typename T> __device__ __forceinline__ const T *fresh(const T *p) {
    int zero = 0;
    asm volatile("" : "+v"(zero));      // opaque: the sum below cannot be computed ahead of the phase
    return p + zero;
}

// RMSNorm of a vector other workgroups wrote, into LDS (K a multiple of 4)
__device__ __forceinline__ void stage_norm_v(float *xs, float *s_red, const float *src, int K, const float *gain, float eps) {
    const int tid = threadIdx.x;
    src = fresh(src); gain = fresh(gain);
    f32x4e_t v[kStageVecs], gn[kStageVecs];
#pragma unroll
    for (int i = 0; i < kStageVecs; ++i) {
        const int k = (tid + i * kFusedThreads) * 4;
        // unconditional (a piece past the end re-reads the last one and is zeroed after the wait): nothing
        // but the wait may touch a result register before its load has landed
        v[i] = ld_coherent4_issue(src + min(k, K - 4));
        gn[i] = *(gptr<f32x4e_t>)(gain + min(k, K - 4));
    }
    coherent_wait(v);
#pragma unroll
    for (int i = 0; i < kStageVecs; ++i)
        if ((tid + i * kFusedThreads) * 4 >= K) v[i] = f32x4e_t{0.f, 0.f, 0.f, 0.f};
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kStageVecs; ++i) ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    ss = wave_sum(ss);
    if ((tid & 63) == 0) s_red[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) tot += s_red[w];
    const float inv = 1.0f / sqrtf(tot / (float)K + eps);
#pragma unroll
    for (int i = 0; i < kStageVecs; ++i) {
        const int k = (tid + i * kFusedThreads) * 4;
        if (k < K) *reinterpret_cast<f32x4e_t *>(xs + k) = v[i] * (gn[i] * inv);
    }
    __syncthreads();
}

__device__ __forceinline__ void stage_copy_v(float *xs, const float *src, int K) {
    const int tid = threadIdx.x;
    src = fresh(src);
    f32x4e_t v[kStageVecs];
#pragma unroll
    for (int i = 0; i < kStageVecs; ++i) {
        const int k = (tid + i * kFusedThreads) * 4;
        v[i] = ld_coherent4_issue(src + min(k, K - 4));     // unconditional, see stage_norm_v
    }
    coherent_wait(v);
#pragma unroll
    for (int i = 0; i < kStageVecs; ++i) {
        const int k = (tid + i * kFusedThreads) * 4;
        if (k < K) *reinterpret_cast<f32x4e_t *>(xs + k) = v[i];
    }
    __syncthreads();
}

// attention output = merge of the per-split partial results (S <= kFusedMaxSplits): a thread takes
// four neighbouring dimensions of a head at a time
template <int HD>
__device__ __forceinline__ void stage_attn_v(float *xs, const float *att_o, const float2 *att_ml, int H, int S) {
    att_o = fresh(att_o); att_ml = fresh(att_ml);
    for (int k = threadIdx.x * 4; k < H * HD; k += kFusedThreads * 4) {
        const int h = k / HD, dd = k % HD;
        f32x4e_t o[kFusedMaxSplits];
        f32x2e_t ml[kFusedMaxSplits];
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s) {
            const int sc = s < S ? s : 0;          // unconditional, see stage_norm_v: a split that does not exist re-reads split 0 ...
            o[s] = ld_coherent4_issue(att_o + ((size_t)h * kFusedMaxSplits + sc) * HD + dd);
            ml[s] = ld_coherent2_issue(att_ml + h * kFusedMaxSplits + sc);
        }
        static_assert(kFusedMaxSplits == 8, "the wait below names eight results");
        coherent_wait(o);
        asm volatile("" : "+v"(ml[0]), "+v"(ml[1]), "+v"(ml[2]), "+v"(ml[3]), "+v"(ml[4]), "+v"(ml[5]), "+v"(ml[6]), "+v"(ml[7]));
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s)
            if (s >= S) ml[s] = f32x2e_t{kNegBig, 0.f};       // ... and gets weight zero
        float M = kNegBig;
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s) M = fmaxf(M, ml[s].x);
        float L = 0.f;
        f32x4e_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s) {
            const float c = __expf(ml[s].x - M);
            L += ml[s].y * c;
            acc += o[s] * c;
        }
        *reinterpret_cast<f32x4e_t *>(xs + k) = acc * (1.0f / L);
    }
    __syncthreads();
}

struct StreamPos { int ri; int nblk; };   // ring position of the next slot; row blocks taken so far (whose turn, which buffer)

// The consuming side of one matrix: NB row blocks of KC tiles, activations staged in xs.
template <int EPI>
__device__ __forceinline__ void stream_rows(const LinArgs<bf16_t> &a, const StreamRing *ring, const float *xs, const float *xzero,
                                            float *red, int NB, int KC, StreamPos &sp, EntStat &st) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = (KC + 7) >> 3;
    const float *xq = xs + (lane >> 4) * 8;
    int pend = -1, pend_wave = 0, pend_par = 0;
    EpiPre pend_pre{};
    auto finish = [&]() {          // the row block `pend`: add the waves' partial sums, run the epilogue
        if (wave == pend_wave && lane < 16) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < kFusedWaves; ++w) v += red[(pend_par * kFusedWaves + w) * 16 + lane];
            epilogue<bf16_t, EPI, true>(a, pend * 16 + lane, 0, v, true, st, pend_pre);
        }
    };
    for (int rb = blockIdx.x; rb < NB; rb += gridDim.x) {
        const int my_wave = sp.nblk & (kFusedWaves - 1), par = sp.nblk & 1;
        // what this row block's epilogue reads is requested now and arrives during its k loop
        const EpiPre pre = epi_prefetch<bf16_t, EPI, true>(a, rb * 16 + (lane & 15), 0, wave == my_wave && lane < 16);
        // A slot's tile and activations are read right behind its barrier and multiplied behind the NEXT
        // one, while the next slot's reads are in flight: the step is then as long as an LDS read, not a
        // read plus a chain of sixteen multiply-adds.  Two sums keep that chain short.
        float acc0 = 0.f, acc1 = 0.f;
        u32x4_t w{};
        float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0;
        auto multiply = [&]() {
            Vec8<bf16_t> t8; t8.raw = w;
            float wf[8];
            t8.unpack_w(wf);
            acc0 += wf[0] * x0.x + wf[1] * x0.y + wf[2] * x0.z + wf[3] * x0.w;
            acc1 += wf[4] * x1.x + wf[5] * x1.y + wf[6] * x1.z + wf[7] * x1.w;
        };
        for (int t = 0; t < nt; ++t) {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const u32x4_t wn = ring[sp.ri][wave][lane];
            sp.ri = sp.ri + 1 == kStreamDepth ? 0 : sp.ri + 1;
            const int kc = t * kFusedWaves + wave;
            const float *xp = kc < KC ? xq + kc * 32 : xzero;
            const float4 xn0 = *reinterpret_cast<const float4 *>(xp);
            const float4 xn1 = *reinterpret_cast<const float4 *>(xp + 4);
            if (t == 0 && pend >= 0) finish();
            if (t > 0) multiply();
            w = wn; x0 = xn0; x1 = xn1;
        }
        multiply();
        float acc = acc0 + acc1;
        acc += __shfl_xor(acc, 16, kWave);
        acc += __shfl_xor(acc, 32, kWave);
        if (lane < 16) red[(par * kFusedWaves + wave) * 16 + lane] = acc;
        pend = rb; pend_wave = my_wave; pend_par = par; pend_pre = pre;
        ++sp.nblk;
    }
    if (pend >= 0) { __syncthreads(); finish(); }     // kSyncRowsEnd
}

template <int HD, int G>
__global__ __launch_bounds__(kStreamThreads) void k_decode_stream(FusedArgs<bf16_t> a, StreamModel sm) {
    typedef bf16_t WT;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    StreamRing *ring = reinterpret_cast<StreamRing *>(smem_raw);
    float *smem = reinterpret_cast<float *>(smem_raw + (size_t)kStreamDepth * kStreamSlotBytes);
    __shared__ int s_plan[4];        // seq, pos, token, T(=1)
    __shared__ int s_ok;
    __shared__ float s_red[kFusedWaves];
    const int Kmax = max(max(a.d, a.F), a.H * HD);
    float *xs = smem, *red = smem + Kmax, *xzero = red + 2 * kFusedWaves * 16;       // xzero: 64 zeros
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long n_steps = stream_steps(sm, blockIdx.x, gridDim.x);

    if (wave >= kFusedWaves) {
        // ---- fetching waves ------------------------------------------------------------------
        const int p = wave - kFusedWaves;
        if (n_steps == 0) { __syncthreads(); return; }
        StreamList pos(sm);
        pos.open();                         // n_steps > 0: there is a first matrix
        int ri = 0;
        for (int s = 0; s < kStreamDepth - 1; ++s) { stream_issue(pos, ring[ri], p, lane); ri = ri + 1 == kStreamDepth ? 0 : ri + 1; }
        __syncthreads();                    // the consuming waves have set up their constants
        // the consuming waves' phases, one by one: arrive where they meet, hand over a slot where they read one
        const int n_phases = 5 * pos.L + 1;
        for (int ph = 0; ph < n_phases; ++ph) {
            const int kind = ph < 5 * pos.L ? ph % 5 : 5;
            if (ph > 0) follow(kSyncGridBarrier);
            if (kind == 1) { follow(kSyncAttention); continue; }
            follow(kind == 2 ? kSyncStageAttn : kind == 4 ? kSyncStageCopy : kSyncStageNorm);
            const int j = kind == 0 ? 0 : kind == 5 ? 4 : kind - 1;
            const int NB = pos.nb_of(j);
            if (pos.wg >= NB) continue;
            const long n = (long)((NB - pos.wg + pos.G - 1) / pos.G) * ((pos.kc_of(j) + 7) >> 3);
            for (long i = 0; i < n; ++i) {
                asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kStreamLoads * (kStreamDepth - 2)) : "memory");
                stream_issue(pos, ring[ri], p, lane);
                ri = ri + 1 == kStreamDepth ? 0 : ri + 1;
            }
            follow(kSyncRowsEnd);
        }
        follow(kSyncGridBarrier);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    // ---- consuming waves -----------------------------------------------------------------------
    if (tid < 64) xzero[tid] = 0.f;
    const int m = a.fin.model_id, MB = a.fin.s.max_batch;
    // the one sequence this model serves in this step, and its newest position
    if (tid == 0) {
        int seq = 0;
        for (int b = 0; b < a.batch; ++b)
            if (!a.fin.s.done[b] && a.fin.s.model[b] == m && a.fin.s.last_step[b] != a.fin.step) { seq = b; break; }
        const int pos = a.fin.s.kvlen[m * MB + seq];
        s_plan[0] = seq; s_plan[1] = pos; s_plan[2] = a.fin.s.tokens[(size_t)seq * a.fin.s.max_seq + pos]; s_plan[3] = 1;
    }
    __syncthreads();
    BlockSync sync;
    StreamPos sp{0, 0};
    const int seq = s_plan[0], pos = s_plan[1];
    const WT *emb = a.embed + (size_t)s_plan[2] * a.d;
    const int NQ = a.H * HD, NK = a.KV * HD;
    // key splits of the attention phase: 64 keys or more each, as many workgroups as that gives
    const int S = min(kFusedMaxSplits, max(1, (pos + 1 + 63) / 64));
    GridBar bar = a.bar;
    EntStat st; st.init();

    // phases: per layer QKV, attention, output projection, gate/up, down; then the LM head.
    // Every workgroup-wide meeting below is counted in the kSync* constants the fetching waves follow.
    const int n_phases = 5 * a.L + 1;
    for (int ph = 0; ph < n_phases; ++ph) {
        const int kind = ph < 5 * a.L ? ph % 5 : 5, l = ph / 5;
        if (ph > 0) {
            bar_arrive(bar, sync);
            if (!bar_wait(bar, &s_ok, sync)) return;
        }
        if (kind == 1) {
            const FusedLayer<WT> ly = a.layers[l];
            if ((int)blockIdx.x < a.KV * S) fused_attention<WT, HD, G>(a, ly.kcache, ly.vcache, seq, pos, S, smem, sync);
            else __syncthreads();
            continue;
        }
        LinArgs<WT> p{};
        if (kind == 0) {                        // RMSNorm + QKV + rotary + KV append
            const FusedLayer<WT> ly = a.layers[l];
            if (l == 0) stage_norm_embed<WT>(xs, s_red, emb, a.d, ly.g_attn, a.eps, sync);
            else stage_norm_v(xs, s_red, a.x, a.d, ly.g_attn, a.eps);
            p.Np = NQ + 2 * NK; p.K = a.d; p.out = a.q; p.ldo = NQ; p.kcache = ly.kcache; p.vcache = ly.vcache; p.vtcache = ly.vtcache;
            p.row_seq = &s_plan[0]; p.row_pos = &s_plan[1]; p.rope = a.rope; p.n_heads = a.H; p.n_kv_heads = a.KV;
            p.hd = HD; p.max_seq = a.fin.s.max_seq;
            stream_rows<EPI_QKV>(p, ring, xs, xzero, red, sm.NB[0], sm.KC[0], sp, st);
        } else if (kind == 2) {                 // output projection + residual
            stage_attn_v<HD>(xs, a.att_o, a.att_ml, a.H, S);
            p.Np = a.d; p.K = NQ; p.out = a.x; p.ldo = a.d; p.res_embed = l == 0 ? emb : nullptr;
            stream_rows<EPI_RES>(p, ring, xs, xzero, red, sm.NB[1], sm.KC[1], sp, st);
        } else if (kind == 3) {                 // RMSNorm + gate/up + SwiGLU
            stage_norm_v(xs, s_red, a.x, a.d, a.layers[l].g_ffn, a.eps);
            p.Np = 2 * a.F; p.K = a.d; p.out = a.hbuf; p.ldo = a.F;
            stream_rows<EPI_SWIGLU>(p, ring, xs, xzero, red, sm.NB[2], sm.KC[2], sp, st);
        } else if (kind == 4) {                 // down projection + residual
            stage_copy_v(xs, a.hbuf, a.F);
            p.Np = a.d; p.K = a.F; p.out = a.x; p.ldo = a.d;
            stream_rows<EPI_RES>(p, ring, xs, xzero, red, sm.NB[3], sm.KC[3], sp, st);
        } else {                                // final RMSNorm + LM head, entropy statistics folded in
            stage_norm_v(xs, s_red, a.x, a.d, a.g_final, a.eps);
            p.Np = a.V; p.K = a.d;
            stream_rows<EPI_LOGITS>(p, ring, xs, xzero, red, sm.NB[4], sm.KC[4], sp, st);
            if (lane < 16) {                    // one partial per (workgroup, wave)
                p.partials = a.lm_part + (size_t)wave * gridDim.x;
                logits_flush<WT, true>(p, 0, true, st);
            }
        }
    }
    bar_arrive(bar, sync);
    if (!bar_wait(bar, &s_ok, sync)) return;
    if (blockIdx.x == 0 && wave == 0) {
        EntStat r; r.init();
        for (int i = lane; i < (int)gridDim.x * kFusedWaves; i += 64) {
            EntStat q;
            q.m = ld_coherent(&a.lm_part[i].m); q.Z = ld_coherent(&a.lm_part[i].Z);
            q.S = ld_coherent(&a.lm_part[i].S); q.idx = ld_coherent(&a.lm_part[i].idx);
            q.gs = -INFINITY; q.gidx = 0x7FFFFFFF;      // this kernel decodes greedily (the host keeps sampled runs off it)
            r.merge(q);
        }
        r = wave_merge(r);
        const float H = entropy_from(r, a.fin.unit);
        if (lane == 0) {
            lm_finalize_seq(a.fin, seq, r, H);
            a.fin.s.kvlen[m * MB + seq] = pos + 1;
        }
    }
}

}  // namespace ead
