// One decode step of one model for a single token row as ONE persistent kernel.
//
// At batch 1 a decoder layer is five dependent, bandwidth-bound phases of a few
// microseconds each (QKV, attention, output projection, gate/up, down).  Launching them
// as separate kernels leaves HBM idle at every boundary.  Here 256 workgroups (one per
// CU, 8 waves each) stay resident for the whole step and meet at grid barriers instead;
// every wave keeps two 8-tile groups of its weight stream in flight (two register buffers
// that take turns) and the stream does not stop at a barrier, so the next phase's weights
// are already on their way (8 waves x 16 KB per CU) while the grid synchronises and the
// activations are re-staged.
// The cursor pauses only in front of the attention phase (whose inputs are the K/V
// cache, not weights).
//
// Work split inside a phase is the same as in k_linear_valu: a workgroup owns 16-row
// blocks wg, wg+G, ... and its waves split K; partial sums meet in LDS in wave order.
#pragma once
#include "attention.hpp"
#include "common.hpp"
#include "linear.hpp"
#include "state.hpp"

namespace ead {

constexpr int kFusedWaves = 8;
constexpr int kFusedThreads = kFusedWaves * 64;
constexpr long kFusedSpinLimit = 1L << 21;
constexpr int kFusedMaxSplits = 8;
constexpr int kBarGroups = 8;
constexpr int kFusedRbChunk = 8;     // row blocks between two workgroup synchronisations
constexpr int kFusedMaxMats = 200;   // 4 per layer + LM head

// ---- grid barrier ---------------------------------------------------------------------
// Counters only grow: `epoch` is the number of barriers passed since they were zeroed
// (the host carries it from launch to launch).  Arrival is counted per group of
// workgroups (wg % 8) so that no single address takes 256 atomics; the last arrival of a
// group bumps the global counter, which everybody polls.  A bounded spin turns a lost
// workgroup into an error flag instead of a hang: every workgroup that sees the flag
// leaves the kernel.
//
// No cache write-back or invalidate is issued: everything one workgroup hands to another
// inside this kernel is written with st_coherent (write-through) and read with
// ld_coherent, so a barrier only has to wait until the stores have completed.  Weights
// and gains are immutable and K/V lines are never read before they are written, so those
// keep using ordinary cached / streaming loads.
struct GridBar { unsigned *grp, *glob; int *abort_flag; unsigned epoch; };

// How the threads that run the phases of a step meet inside their workgroup.  Here: all of them, at
// the hardware barrier.  The streamed kernel passes a policy of its own, because there the
// hardware barrier belongs to the weight stream.
struct BlockSync { __device__ __forceinline__ void operator()() const { __syncthreads(); } };

template <typename Sync>
__device__ __forceinline__ void bar_arrive(GridBar &b, Sync &sync) {
    wait_stores();
    sync();
    b.epoch++;
    if (threadIdx.x == 0) {
        const unsigned g = blockIdx.x % kBarGroups;
        const unsigned gsize = (gridDim.x - g + kBarGroups - 1) / kBarGroups;
        const unsigned old = __hip_atomic_fetch_add(b.grp + g * 32, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == b.epoch * gsize) __hip_atomic_fetch_add(b.glob, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// returns false when the barrier was abandoned
template <typename Sync>
__device__ __forceinline__ bool bar_wait(GridBar &b, int *s_ok, Sync &sync) {
    if (threadIdx.x == 0) {
        const unsigned target = b.epoch * kBarGroups;
        long spins = 0;
        int ok = 1;
        while ((int)(__hip_atomic_load(b.glob, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            if (++spins > kFusedSpinLimit || __hip_atomic_load(b.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                __hip_atomic_store(b.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        *s_ok = ok;
    }
    sync();
    return *s_ok != 0;
}

// ---- model description on the device ------------------------------------------------------
template <typename WT>
struct FusedMat { const WT *W; int NB, KC; int stop_after; };   // stop_after: cursor pauses behind it

template <typename WT>
struct FusedLayer { const float *g_attn, *g_ffn; WT *kcache, *vcache, *vtcache; };

template <typename WT>
struct FusedArgs {
    int L, d, H, KV, hd, F, V;
    float eps;
    const FusedMat<WT> *mats;        // 4 per layer (qkv, wo, gate/up, down) + LM head
    const FusedLayer<WT> *layers;
    const WT *embed;
    const float *g_final;
    const float2 *rope;
    float *x, *q, *hbuf;             // [d], [H*hd], [F]
    float *att_o; float2 *att_ml;    // [H][kFusedMaxSplits][hd], [H][kFusedMaxSplits]
    EntPartial *lm_part;             // [gridDim.x]
    GridBar bar;
    FinArgs fin;
    int batch, n_mats;
};

// ---- staging the activation vector of a phase into LDS ----------------------------------------
// Right after a grid barrier every one of these loads misses the caches, so all loads of a
// thread are issued before the first use (K <= 16384: at most 32 per thread).  Vectors
// written by other workgroups during this kernel are read with ld_coherent.
constexpr int kStageElems = 32;      // elements per thread: K <= 32 * 512

template <typename Sync>
__device__ __forceinline__ void stage_norm(float *xs, float *s_red, const float *src, int K, const float *gain, float eps, Sync &sync) {
    const int tid = threadIdx.x;
    float v[kStageElems], gn[kStageElems];
#pragma unroll
    for (int i = 0; i < kStageElems; ++i) {
        const int k = tid + i * kFusedThreads;
        if (k < K) { v[i] = ld_coherent(src + k); gn[i] = gain[k]; } else { v[i] = 0.f; gn[i] = 0.f; }
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kStageElems; ++i) ss += v[i] * v[i];
    ss = wave_sum(ss);
    if ((tid & 63) == 0) s_red[tid >> 6] = ss;
    sync();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) tot += s_red[w];
    const float inv = 1.0f / sqrtf(tot / (float)K + eps);
#pragma unroll
    for (int i = 0; i < kStageElems; ++i) {
        const int k = tid + i * kFusedThreads;
        if (k < K) xs[k] = v[i] * (inv * gn[i]);
    }
    sync();
}

// first layer: the residual stream is the embedding row itself
template <typename ST, typename Sync>
__device__ __forceinline__ void stage_norm_embed(float *xs, float *s_red, const ST *src, int K, const float *gain, float eps, Sync &sync) {
    const int tid = threadIdx.x;
    float ss = 0.f;
    for (int k = tid; k < K; k += kFusedThreads) { const float v = to_f32(src[k]); xs[k] = v; ss += v * v; }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) s_red[tid >> 6] = ss;
    sync();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) tot += s_red[w];
    const float inv = 1.0f / sqrtf(tot / (float)K + eps);
    for (int k = tid; k < K; k += kFusedThreads) xs[k] *= inv * gain[k];
    sync();
}

template <typename Sync>
__device__ __forceinline__ void stage_copy(float *xs, const float *src, int K, Sync &sync) {
    const int tid = threadIdx.x;
    float v[kStageElems];
#pragma unroll
    for (int i = 0; i < kStageElems; ++i) {
        const int k = tid + i * kFusedThreads;
        if (k < K) v[i] = ld_coherent(src + k);
    }
#pragma unroll
    for (int i = 0; i < kStageElems; ++i) {
        const int k = tid + i * kFusedThreads;
        if (k < K) xs[k] = v[i];
    }
    sync();
}

// attention output = merge of the per-split partial results (S <= kFusedMaxSplits)
template <typename Sync>
__device__ __forceinline__ void stage_attn(float *xs, const float *att_o, const float2 *att_ml, int H, int hd, int S, Sync &sync) {
    for (int k = threadIdx.x; k < H * hd; k += kFusedThreads) {
        const int h = k / hd, dd = k % hd;
        float mm[kFusedMaxSplits], ll[kFusedMaxSplits], o[kFusedMaxSplits];
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s) {
            if (s < S) {
                const float *ml = reinterpret_cast<const float *>(att_ml + h * kFusedMaxSplits + s);
                mm[s] = ld_coherent(ml); ll[s] = ld_coherent(ml + 1);
                o[s] = ld_coherent(att_o + ((size_t)h * kFusedMaxSplits + s) * hd + dd);
            } else { mm[s] = kNegBig; ll[s] = 0.f; o[s] = 0.f; }
        }
        float M = kNegBig;
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s) M = fmaxf(M, mm[s]);
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int s = 0; s < kFusedMaxSplits; ++s) {
            const float c = __expf(mm[s] - M);
            L += ll[s] * c;
            acc += o[s] * c;
        }
        xs[k] = acc / L;
    }
    sync();
}

// ---- one linear phase --------------------------------------------------------------------------
// The weight stream of a wave is the concatenation, over the matrices of the step in which
// its workgroup owns row blocks, of its K-slice of the row blocks wg, wg+G, ...  It is read
// in groups of U tiles.  Two register buffers take turns: while one group is multiplied the
// other is in flight, and as soon as a group has been multiplied the group after next is
// requested into the same registers -- also across the end of a matrix, so that the first
// two groups of the next phase are on their way while the grid synchronises.  Control is
// wave-uniform and the loads are unconditional (tiles past the end of a slice re-read its
// last tile and meet zeros), which keeps a group step free of branches around the loads.
template <typename WT>
struct WaveSlice {                   // this wave's share of one matrix
    const WT *W; int NB, KC, kc0, kc1, ng;
    __device__ __forceinline__ void set(const FusedMat<WT> &m, int wave) {
        constexpr int U = sizeof(WT) == 2 ? 8 : 4;
        // descriptors come from LDS: tell the compiler they are the same in every lane
        const uint64_t w = (uint64_t)m.W;
        const uint32_t w_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(w >> 32));
        const uint32_t w_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)w);   // no sign extension
        W = (const WT *)(((uint64_t)w_hi << 32) | (uint64_t)w_lo);
        NB = __builtin_amdgcn_readfirstlane(m.NB); KC = __builtin_amdgcn_readfirstlane(m.KC);
        kc0 = (wave * KC) / kFusedWaves; kc1 = ((wave + 1) * KC) / kFusedWaves;
        ng = ((KC + kFusedWaves - 1) / kFusedWaves + U - 1) / U;
    }
};

template <typename WT, int U>
__device__ __forceinline__ void issue_group(Vec8<WT> (&buf)[U], const WT *W, int KC, int rb, int kc, int kc1, int lane) {
    const WT *base = W + tile_offset(rb, 0, KC) + lane * 8;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = max(min(kc + u, kc1 - 1), 0);
        buf[u].load_stream(base + (size_t)t * 512);
    }
}

// Walks the wave's stream two groups ahead of the arithmetic.
template <typename WT>
struct IssueCursor {
    static constexpr int U = sizeof(WT) == 2 ? 8 : 4;
    const FusedMat<WT> *mats; int n_mats, im, wave, lane;
    WaveSlice<WT> s; int rb, gi;
    bool none, done;                 // none: no matrix has a row block for this workgroup
    __device__ __forceinline__ int next_owned(int j) const {
        while (j < n_mats && (int)blockIdx.x >= __builtin_amdgcn_readfirstlane(mats[j].NB)) ++j;
        return j;
    }
    __device__ __forceinline__ void init(const FusedMat<WT> *m, int n, int wave_, int lane_) {
        mats = m; n_mats = n; wave = wave_; lane = lane_; done = false;
        im = next_owned(0); none = im >= n_mats;
        if (!none) { s.set(mats[im], wave); rb = blockIdx.x; gi = 0; }
    }
    __device__ __forceinline__ void issue(Vec8<WT> (&buf)[U]) {
        if (none) return;
        issue_group<WT, U>(buf, s.W, s.KC, rb, s.kc0 + gi * U, s.kc1, lane);
        if (done) return;                                   // past the end: keep re-reading the last group
        if (++gi == s.ng) {
            gi = 0; rb += gridDim.x;
            if (rb >= s.NB) {
                const int j = next_owned(im + 1);
                if (j < n_mats) { im = j; s.set(mats[j], wave); rb = blockIdx.x; }
                else { done = true; rb -= gridDim.x; gi = s.ng - 1; }
            }
        }
    }
};

// One group step: multiply the group in `buf`, then request the group after next into it.
template <typename WT, int U>
__device__ __forceinline__ float group_step(Vec8<WT> (&buf)[U], IssueCursor<WT> &ic, const float *xq, const float *xzero,
                                            int kc, int kc1) {
    float part = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float wf[8];
        buf[u].unpack_w(wf);
        const float *xp = (kc + u < kc1) ? xq + (kc + u) * 32 : xzero;
        const float4 x0 = *reinterpret_cast<const float4 *>(xp);
        const float4 x1 = *reinterpret_cast<const float4 *>(xp + 4);
        part += wf[0] * x0.x + wf[1] * x0.y + wf[2] * x0.z + wf[3] * x0.w
              + wf[4] * x1.x + wf[5] * x1.y + wf[6] * x1.z + wf[7] * x1.w;
    }
    // neither the scheduler nor code sinking may move the refill above the arithmetic (it
    // would need a third buffer): pin the sum here
    asm volatile("" : "+v"(part));
    __builtin_amdgcn_sched_barrier(0);
    ic.issue(buf);
    __builtin_amdgcn_sched_barrier(0);
    return part;
}

// The groups of up to kFusedRbChunk row blocks; X holds the first group, Y the second.
// Returns true when an odd number of groups was taken (the buffers have swapped roles).
template <typename WT>
__device__ __forceinline__ bool chunk_groups(Vec8<WT> (&X)[sizeof(WT) == 2 ? 8 : 4], Vec8<WT> (&Y)[sizeof(WT) == 2 ? 8 : 4],
                                             IssueCursor<WT> &ic, const WaveSlice<WT> &cs, int nin, const float *xq,
                                             const float *xzero, float *red, int wave, int lane) {
    constexpr int U = sizeof(WT) == 2 ? 8 : 4;
    const int n = nin * cs.ng;
    int gi = 0, slot = 0, i = 0;
    float acc = 0.f;
    auto end_of_group = [&]() {
        if (++gi == cs.ng) {                 // last group of a row block: leave the partial sums in LDS
            gi = 0;
            acc += __shfl_xor(acc, 16, kWave);
            acc += __shfl_xor(acc, 32, kWave);
            if (lane < 16) red[(slot * kFusedWaves + wave) * 16 + lane] = acc;
            acc = 0.f; ++slot;
        }
    };
    for (; i + 2 <= n; i += 2) {
        acc += group_step<WT, U>(X, ic, xq, xzero, cs.kc0 + gi * U, cs.kc1);
        end_of_group();
        acc += group_step<WT, U>(Y, ic, xq, xzero, cs.kc0 + gi * U, cs.kc1);
        end_of_group();
    }
    if (i < n) {
        acc += group_step<WT, U>(X, ic, xq, xzero, cs.kc0 + gi * U, cs.kc1);
        end_of_group();
        return true;
    }
    return false;
}

template <typename WT>
__device__ __forceinline__ void fused_linear(const LinArgs<WT> &a, int epi, const float *xs, const float *xzero,
                                             float *red, const WaveSlice<WT> &cs, IssueCursor<WT> &ic,
                                             Vec8<WT> (&A)[sizeof(WT) == 2 ? 8 : 4], Vec8<WT> (&B)[sizeof(WT) == 2 ? 8 : 4],
                                             int &par, EntStat &st) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 4;
    const int G = gridDim.x;
    const float *xq = xs + g * 8;
    // Row blocks are taken kFusedRbChunk at a time: each wave leaves its partial sums in LDS
    // and moves on, and the workgroup synchronises once per chunk, so the waves of a CU
    // drift apart and keep their loads evenly in flight.
    for (int rb0 = blockIdx.x; rb0 < cs.NB; rb0 += G * kFusedRbChunk) {
        const int nin = min(kFusedRbChunk, (cs.NB - rb0 + G - 1) / G);
        const bool flipped = par ? chunk_groups<WT>(B, A, ic, cs, nin, xq, xzero, red, wave, lane)
                                 : chunk_groups<WT>(A, B, ic, cs, nin, xq, xzero, red, wave, lane);
        par ^= flipped ? 1 : 0;
        __syncthreads();
        if (tid < 16 * nin) {
            const int i = tid >> 4, j = tid & 15;
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < kFusedWaves; ++w) v += red[(i * kFusedWaves + w) * 16 + j];
            const int p = (rb0 + i * G) * 16 + j;
            switch (epi) {
                case EPI_QKV: epilogue<WT, EPI_QKV, true>(a, p, 0, v, true, st, epi_prefetch<WT, EPI_QKV, true>(a, p, 0, true)); break;
                case EPI_RES: epilogue<WT, EPI_RES, true>(a, p, 0, v, true, st, epi_prefetch<WT, EPI_RES, true>(a, p, 0, true)); break;
                case EPI_SWIGLU: epilogue<WT, EPI_SWIGLU, true>(a, p, 0, v, true, st, epi_prefetch<WT, EPI_SWIGLU, true>(a, p, 0, true)); break;
                default: epilogue<WT, EPI_LOGITS, true>(a, p, 0, v, true, st, epi_prefetch<WT, EPI_LOGITS, true>(a, p, 0, true)); break;
            }
        }
        __syncthreads();
    }
}

// ---- attention of the single query row, split over workgroups and their waves ------------------
// Workgroup = (KV head, key split).  Inside it every wave serves ONE of the G query heads
// of that KV head on one slice of the split's keys (wave w: head w % G, slice w / G), so
// the per-lane state is one head's worth; the waves' results meet in LDS and the
// workgroup writes one un-normalised partial per head for stage_attn to merge.
template <typename KT, int HD, int G, typename Sync>
__device__ __forceinline__ void fused_attention(const FusedArgs<KT> &a, const KT *kcache, const KT *vcache, int seq,
                                                int pos, int S, float *lds, Sync &sync) {
    constexpr int LPK = HD / 8, KPI = 64 / LPK, NI = 4, CH = NI * KPI;
    constexpr int NS = kFusedWaves / G;            // key slices per workgroup
    const int item = blockIdx.x;
    if (item >= a.KV * S) return;
    const int kvh = item / S, split = item % S;
    const int nkeys = pos + 1;
    const int per = (nkeys + S - 1) / S;
    const int k0 = split * per, k1 = min(k0 + per, nkeys);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = lane / LPK, dl = lane % LPK;
    const int g = wave % G, slice = wave / G;
    const bool active = slice < NS;
    const float scale = 1.0f / sqrtf((float)HD);
    float qv[8], o[8], m = kNegBig, l = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { qv[e] = ld_coherent(a.q + (size_t)(kvh * G + g) * HD + dl * 8 + e) * scale; o[e] = 0.f; }
    const size_t base = ((size_t)seq * a.KV + kvh) * (size_t)a.fin.s.max_seq * HD;
    const KT *kb = kcache + base + dl * 8, *vb = vcache + base + dl * 8;
    if (active) {
        for (int c0 = k0 + slice * CH; c0 < k1; c0 += NS * CH) {
            Vec8<KT> kx[NI], vx[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int kk = c0 + i * KPI + slot;
                if (kk < k1) { kx[i].load(kb + (size_t)kk * HD); vx[i].load(vb + (size_t)kk * HD); }
                else { kx[i].zero(); vx[i].zero(); }
            }
            float s[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                float kf[8];
                kx[i].unpack(kf);
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d += qv[e] * kf[e];
#pragma unroll
                for (int off = 1; off < LPK; off <<= 1) d += __shfl_xor(d, off, kWave);
                s[i] = (c0 + i * KPI + slot < k1) ? d : kNegBig;
            }
            float mc = s[0];
#pragma unroll
            for (int i = 1; i < NI; ++i) mc = fmaxf(mc, s[i]);
            const float mn = fmaxf(m, mc);
            const float corr = __expf(m - mn);
            l *= corr;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] *= corr;
            m = mn;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const float p = (c0 + i * KPI + slot < k1) ? __expf(s[i] - mn) : 0.f;
                l += p;
                float vf[8];
                vx[i].unpack(vf);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += p * vf[e];
            }
        }
    }
    // merge the key slots of the wave
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m, off, kWave), l2 = __shfl_xor(l, off, kWave);
        const float M = fmaxf(m, m2);
        const float ca = __expf(m - M), cb = __expf(m2 - M);
        l = l * ca + l2 * cb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float o2 = __shfl_xor(o[e], off, kWave);
            o[e] = o[e] * ca + o2 * cb;
        }
        m = M;
    }
    // waves meet in LDS: wo[wave][HD], wm[wave], wl[wave]
    float *wo = lds, *wm = lds + kFusedWaves * HD, *wl = wm + kFusedWaves;
    if (slot == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) wo[wave * HD + dl * 8 + e] = o[e];
        if (dl == 0) { wm[wave] = active ? m : kNegBig; wl[wave] = active ? l : 0.f; }
    }
    sync();
    for (int e = tid; e < G * HD; e += kFusedThreads) {
        const int gg = e / HD, dd = e % HD;
        float M = kNegBig;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) M = fmaxf(M, wm[sl * G + gg]);
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            const float c = __expf(wm[sl * G + gg] - M);
            L += wl[sl * G + gg] * c;
            acc += wo[(sl * G + gg) * HD + dd] * c;
        }
        const int h = kvh * G + gg;
        st_coherent(a.att_o + ((size_t)h * kFusedMaxSplits + split) * HD + dd, acc);
        if (dd == 0) {
            float *ml = reinterpret_cast<float *>(a.att_ml + h * kFusedMaxSplits + split);
            st_coherent(ml, M); st_coherent(ml + 1, L);
        }
    }
}

// ---- the kernel ------------------------------------------------------------------------------------
template <typename WT, int HD, int G>
__global__ __launch_bounds__(kFusedThreads) void k_decode_fused(FusedArgs<WT> a) {
    constexpr int U = sizeof(WT) == 2 ? 8 : 4;
    extern __shared__ float smem[];
    __shared__ int s_plan[4];        // seq, pos, token, T(=1)
    __shared__ int s_ok;
    __shared__ float s_red[kFusedWaves];
    const int Kmax = max(max(a.d, a.F), a.H * HD);
    float *xs = smem, *red = smem + Kmax, *xzero = red + kFusedRbChunk * kFusedWaves * 16;   // xzero: 64 zeros
    BlockSync sync;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = a.fin.model_id, MB = a.fin.s.max_batch;

    __shared__ FusedMat<WT> s_mats[kFusedMaxMats];
    for (int i = tid; i < a.n_mats; i += kFusedThreads) s_mats[i] = a.mats[i];
    if (tid < 64) xzero[tid] = 0.f;
    __syncthreads();
    IssueCursor<WT> ic;
    ic.init(s_mats, a.n_mats, wave, lane);
    Vec8<WT> A[U], B[U];
    int par = 0;                                // 0: the next group to multiply is in A
    ic.issue(A);
    ic.issue(B);
    WaveSlice<WT> cs;

    // the one sequence this model serves in this step, and its newest position
    if (tid == 0) {
        int seq = 0;
        for (int b = 0; b < a.batch; ++b)
            if (!a.fin.s.done[b] && a.fin.s.model[b] == m && a.fin.s.last_step[b] != a.fin.step) { seq = b; break; }
        const int pos = a.fin.s.kvlen[m * MB + seq];
        s_plan[0] = seq; s_plan[1] = pos; s_plan[2] = a.fin.s.tokens[(size_t)seq * a.fin.s.max_seq + pos]; s_plan[3] = 1;
    }
    __syncthreads();
    const int seq = s_plan[0], pos = s_plan[1];
    const WT *emb = a.embed + (size_t)s_plan[2] * a.d;
    const int NQ = a.H * HD, NK = a.KV * HD;
    const int S = min(kFusedMaxSplits, max(1, (pos + 1 + 255) / 256));
    GridBar bar = a.bar;
    EntStat st; st.init();

    // phases: per layer QKV, attention, output projection, gate/up, down; then the LM head
    const int n_phases = 5 * a.L + 1;
    for (int ph = 0; ph < n_phases; ++ph) {
        const int kind = ph < 5 * a.L ? ph % 5 : 5, l = ph / 5;
        if (ph > 0) {
            bar_arrive(bar, sync);
            if (!bar_wait(bar, &s_ok, sync)) return;
        }
        if (kind == 1) {
            const FusedLayer<WT> ly = a.layers[l];
            fused_attention<WT, HD, G>(a, ly.kcache, ly.vcache, seq, pos, S, smem, sync);
            continue;
        }
        LinArgs<WT> p{};
        int epi;
        if (kind == 0) {                        // RMSNorm + QKV + rotary + KV append
            const FusedLayer<WT> ly = a.layers[l];
            if (l == 0) stage_norm_embed<WT>(xs, s_red, emb, a.d, ly.g_attn, a.eps, sync);
            else stage_norm(xs, s_red, a.x, a.d, ly.g_attn, a.eps, sync);
            epi = EPI_QKV;
            p.Np = NQ + 2 * NK; p.K = a.d; p.out = a.q; p.ldo = NQ; p.kcache = ly.kcache; p.vcache = ly.vcache; p.vtcache = ly.vtcache;
            p.row_seq = &s_plan[0]; p.row_pos = &s_plan[1]; p.rope = a.rope; p.n_heads = a.H; p.n_kv_heads = a.KV;
            p.hd = HD; p.max_seq = a.fin.s.max_seq;
        } else if (kind == 2) {                 // output projection + residual
            stage_attn(xs, a.att_o, a.att_ml, a.H, HD, S, sync);
            epi = EPI_RES;
            p.Np = a.d; p.K = NQ; p.out = a.x; p.ldo = a.d; p.res_embed = l == 0 ? emb : nullptr;
        } else if (kind == 3) {                 // RMSNorm + gate/up + SwiGLU
            stage_norm(xs, s_red, a.x, a.d, a.layers[l].g_ffn, a.eps, sync);
            epi = EPI_SWIGLU;
            p.Np = 2 * a.F; p.K = a.d; p.out = a.hbuf; p.ldo = a.F;
        } else if (kind == 4) {                 // down projection + residual
            stage_copy(xs, a.hbuf, a.F, sync);
            epi = EPI_RES;
            p.Np = a.d; p.K = a.F; p.out = a.x; p.ldo = a.d;
        } else {                                // final RMSNorm + LM head, entropy statistics folded in
            stage_norm(xs, s_red, a.x, a.d, a.g_final, a.eps, sync);
            epi = EPI_LOGITS;
            p.Np = a.V; p.K = a.d; p.partials = a.lm_part;
        }
        const int mat = ph < 5 * a.L ? 4 * l + (kind == 0 ? 0 : kind - 1) : 4 * a.L;
        if ((int)blockIdx.x < __builtin_amdgcn_readfirstlane(s_mats[mat].NB)) {     // this workgroup has row blocks here
            cs.set(s_mats[mat], wave);
            fused_linear<WT>(p, epi, xs, xzero, red, cs, ic, A, B, par, st);
        }
        if (kind == 5 && tid < 16 * kFusedRbChunk) {      // one partial per (workgroup, chunk slot)
            p.partials = a.lm_part + (size_t)(tid >> 4) * gridDim.x;
            logits_flush<WT, true>(p, 0, true, st);
        }
    }
    bar_arrive(bar, sync);
    if (!bar_wait(bar, &s_ok, sync)) return;
    if (blockIdx.x == 0 && wave == 0) {
        EntStat r; r.init();
        for (int i = lane; i < (int)gridDim.x * kFusedRbChunk; i += 64) {
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
