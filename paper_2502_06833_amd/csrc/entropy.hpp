// Entropy of the next-token distribution (Eq. 1-2), arg max, rolling window (Eq. 3)
// and the switch rule (Eq. 4 / Algorithm 1's switching block).
#pragma once
#include "common.hpp"
#include "linear.hpp"

namespace ead {

constexpr float kLn2Inv = 1.4426950408889634f;
constexpr int kGateMaxSteps = 16;       // steps of the gate one launch can take

// H = ln Z - S/Z in nats, or divided by ln 2 for bits
__device__ __forceinline__ float entropy_from(const EntStat &s, int unit) {
    float H = logf(s.Z) - s.S / s.Z;
    return unit ? H * kLn2Inv : H;
}

// Merge n partials of one row in a fixed order (lane i takes i, i+64, ...; then the
// wave tree).  Every lane returns the merged statistics.
__device__ __forceinline__ EntStat merge_partials(const EntPartial *p, int n) {
    EntStat st; st.init();
    for (int i = threadIdx.x & 63; i < n; i += 64) {
        EntStat q; q.m = p[i].m; q.Z = p[i].Z; q.S = p[i].S; q.idx = p[i].idx; q.gs = p[i].gs; q.gidx = p[i].gidx;
        st.merge(q);
    }
    return wave_merge(st);
}

// ---------------------------------------------------------------------------------------
// Rolling window + switch rule for one sequence.  Ring buffer of w entropies; the mean is
// re-summed oldest to newest in fp32 every step (no running sum), as the definition reads.
// ---------------------------------------------------------------------------------------
struct GateCfg { int w; float tau; int d_min; };

// n = entropies recorded before this one.  Returns the window mean; updates *model and *c.
__device__ __forceinline__ float gate_update(float *ring, int n, float H, const GateCfg &cfg,
                                             int *model, int *c) {
    ring[n % cfg.w] = H;
    const int cnt = min(n + 1, cfg.w);
    float s = 0.f;
    for (int q = 0; q < cnt; ++q) s = s + ring[(n + 1 - cnt + q) % cfg.w];
    const float Hbar = s / (float)cnt;
    int cc = *c + 1, mm = *model;
    if (cc >= cfg.d_min) {
        if (mm == 0 && Hbar > cfg.tau) { mm = 1; cc = 0; }
        else if (mm == 1 && Hbar <= cfg.tau) { mm = 0; cc = 0; }
    }
    *model = mm; *c = cc;
    return Hbar;
}

struct GateState {           // device arrays, one entry per sequence
    float *ring;             // [rows][w]
    int *n, *c, *model;
};

struct GateStepArgs {
    GateState st; GateCfg cfg; int rows;
    int steps;                      // consecutive steps handled by one launch (partials / outputs strided by rows)
    const float *H;                 // [rows] or null (then from partials)
    const EntPartial *partials; int n_part; int unit;
    float *H_out; int *argmax_out;
    uint8_t *model_id_out; float *Hbar_out; uint8_t *next_out;
};

// A row's window means and switch decisions for the steps of one launch, once their entropies are in
// s_H[0 .. steps) (LDS): called by a whole workgroup of any size; ends with a workgroup barrier.
// s_hb: kGateMaxSteps floats, s_ring: at least cfg.w floats of LDS.
__device__ __forceinline__ void gate_row_apply(const GateStepArgs &a, int r, const float *s_H, float *s_ring, float *s_hb) {
    // the window lives in LDS while the steps are taken: a store-then-load round trip through
    // device memory per step would dominate
    for (int i = threadIdx.x; i < a.cfg.w; i += blockDim.x) s_ring[i] = a.st.ring[(size_t)r * a.cfg.w + i];
    __syncthreads();
    // Window means of all steps side by side (thread s: step s), each summed oldest to newest
    // as the definition reads: entropy number g of the row is s_H[g - n] if this launch
    // produced it, else still in the ring.  Only the switch rule itself is sequential.
    const int n = a.st.n[r], w = a.cfg.w;
    if ((int)threadIdx.x < a.steps) {
        const int g1 = n + (int)threadIdx.x, cnt = min(g1 + 1, w);
        float sum = 0.f;
        for (int g = g1 - cnt + 1; g <= g1; ++g) sum = sum + (g >= n ? s_H[g - n] : s_ring[g % w]);
        s_hb[threadIdx.x] = sum / (float)cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int model = a.st.model[r], c = a.st.c[r];
        for (int s = 0; s < a.steps; ++s) {
            const size_t o = (size_t)s * a.rows + r;
            if (a.model_id_out) a.model_id_out[o] = (uint8_t)model;
            const float hb = s_hb[s];
            ++c;
            if (c >= a.cfg.d_min) {
                if (model == 0 && hb > a.cfg.tau) { model = 1; c = 0; }
                else if (model == 1 && hb <= a.cfg.tau) { model = 0; c = 0; }
            }
            if (a.Hbar_out) a.Hbar_out[o] = hb;
            if (a.next_out) a.next_out[o] = (uint8_t)model;
        }
        a.st.model[r] = model; a.st.c[r] = c; a.st.n[r] = n + a.steps;
    }
    // the ring keeps the last w entropies: slots of the newest min(steps, w) are distinct
    for (int s = max(0, a.steps - w) + (int)threadIdx.x; s < a.steps; s += blockDim.x)
        a.st.ring[(size_t)r * w + (n + s) % w] = s_H[s];
    __syncthreads();
}

// ---------------------------------------------------------------------------------------
// Stand-alone pass over logits matrices [rows, V].  A work item is one chunk of one row of
// one step (up to 2048 vectors of 8 logits); item i leaves partial i.  The grid is
// persistent: a workgroup of 256 threads takes items i, i + grid, ... and keeps loads in
// flight across them -- each thread holds two sets of four vectors, and while it works on
// one set the other (the second half of this item, or the first half of the next) is on
// its way, so memory and arithmetic overlap inside every wave instead of by luck between
// waves.
//
// Two bytes per logit leave only a handful of ALU operations per element before the kernel
// stops being bandwidth-bound, so the work per logit is pared down:
//  * the maximum of a set of 32 logits is found first, then they are exponentiated: one
//    rescale of the running sums per set, not per element;
//  * exponentials are taken in base 2 (the hardware instruction): d = (l - m) log2 e is
//    one FMA, Z = sum 2^d, S2 = sum 2^d d, and S = S2 ln 2 once per item;
//  * d is clamped at -160, where 2^d is 0 in fp32, so -inf logits need no test, and a
//    vector past the end of the chunk is switched off through its FMA offset (-inf);
//  * for the arg max a thread keeps the packed vector that holds its running maximum; the
//    element is looked up at the end, only by the threads that hold the item's maximum.
// ---------------------------------------------------------------------------------------
template <typename T>
struct EntArgs {
    const T *step_logits[kGateMaxSteps];      // one [rows, V] matrix per step of the launch
    int V, rows, chunks, vec_per_item, items; // items = steps * rows * chunks
    EntPartial *partials;                     // [items]
};

constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
constexpr float kEntNone = -1e30f;            // running maximum before any logit was seen

template <typename T>
struct EntItem { const T *base; int v0, v1; };

template <typename T>
__device__ __forceinline__ EntItem<T> ent_item(const EntArgs<T> &a, int item) {
    const int chunk = item % a.chunks, rz = item / a.chunks, row = rz % a.rows, z = rz / a.rows;
    const T *p = a.step_logits[z];
    EntItem<T> it;
    it.base = p + (size_t)row * a.V;
    it.v0 = chunk * a.vec_per_item;
    it.v1 = min(it.v0 + a.vec_per_item, a.V >> 3);
    return it;
}

// vectors j0 .. j0+3 of a thread (vector v0 + tid + 256 j); past the end: a valid address
// whose contents are ignored, so no branch surrounds the loads
template <typename T>
__device__ __forceinline__ void ent_load4(Vec8<T> (&s)[4], const EntItem<T> &it, int j0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = max(min(it.v0 + (int)threadIdx.x + (j0 + i) * 256, it.v1 - 1), 0);
        s[i].load_stream(it.base + (size_t)v * 8);
    }
}

template <typename T>
struct EntRun {              // a thread's running statistics within one item (or one whole row)
    float m, Z, S2; int bestv; Vec8<T> best;      // bestv: index (in vectors of 8 from the row's start) of the vector that holds m
};

template <typename T>
__device__ __forceinline__ void ent_take4(const Vec8<T> (&s)[4], EntRun<T> &r, const EntItem<T> &it, int j0) {
    float f[4][8];
    bool valid[4];
    const float m_old = r.m;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s[i].unpack(f[i]);
        valid[i] = it.v0 + (int)threadIdx.x + (j0 + i) * 256 < it.v1;
        float vm = fmaxf(fmaxf(fmaxf(f[i][0], f[i][1]), fmaxf(f[i][2], f[i][3])),
                         fmaxf(fmaxf(f[i][4], f[i][5]), fmaxf(f[i][6], f[i][7])));
        vm = valid[i] ? vm : kEntNone;
        if (vm > r.m) { r.m = vm; r.bestv = it.v0 + (int)threadIdx.x + (j0 + i) * 256; r.best = s[i]; }
    }
    // move the sums to the new maximum: d' = d - delta
    const float delta = (r.m - m_old) * kLog2e;
    const float sc = __builtin_amdgcn_exp2f(-fminf(delta, 160.f));
    r.S2 = sc * (r.S2 - delta * r.Z);
    r.Z *= sc;
    const float off = -r.m * kLog2e;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float o = valid[i] ? off : -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float d = fmaxf(fmaf(f[i][e], kLog2e, o), -160.f);
            const float ex = __builtin_amdgcn_exp2f(d);
            r.Z += ex;
            r.S2 = fmaf(ex, d, r.S2);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_entropy_partial(EntArgs<T> a) {
    __shared__ float s_max[4];
    __shared__ EntPartial s_fin[4];
    const int tid = threadIdx.x;
    int item = blockIdx.x;                  // uniform: kept in scalar registers
    if (item >= a.items) return;
    EntItem<T> it = ent_item(a, item);
    Vec8<T> A[4], B[4], C[4];
    ent_load4(A, it, 0);
    // one item: `first` holds its first half (already requested), B takes its second half and
    // `next` the first half of the item after it.  Returns true after the last item.
    auto one_item = [&](Vec8<T> (&first)[4], Vec8<T> (&next)[4]) __attribute__((always_inline)) -> bool {
        ent_load4(B, it, 4);
        // the next item's first half is requested before this item's second half is worked
        // on; after the last item the request repeats this one and its result is dropped
        const int nitem = item + gridDim.x;
        const bool more = nitem < a.items;
        const EntItem<T> nit = ent_item(a, more ? nitem : item);
        EntRun<T> r; r.m = kEntNone; r.Z = 0.f; r.S2 = 0.f; r.bestv = 0; r.best.zero();
        // pin the order: without it the compiler moves the next requests behind the second
        // half's arithmetic and nothing is in flight while a wave computes
        __builtin_amdgcn_sched_barrier(0);
        ent_take4(first, r, it, 0);
        __builtin_amdgcn_sched_barrier(0);
        ent_load4(next, nit, 0);
        __builtin_amdgcn_sched_barrier(0);
        ent_take4(B, r, it, 4);

        // the item's maximum; every thread moves its sums to that reference once, so the
        // rest of the reduction is plain sums in a fixed order
        const float wmx = wave_max(r.m);
        if ((tid & 63) == 0) s_max[tid >> 6] = wmx;
        __syncthreads();
        const float gmx = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
        const float delta = (gmx - r.m) * kLog2e;
        const float sc = __builtin_amdgcn_exp2f(-fminf(delta, 160.f));
        float S2 = sc * (r.S2 - delta * r.Z), Z = r.Z * sc;
        int idx = 0x7FFFFFFF;
        if (r.m == gmx && r.m > kEntNone) {
            float f[8];
            r.best.unpack(f);
            int e0 = 8;
#pragma unroll
            for (int e = 7; e >= 0; --e) if (f[e] == r.m) e0 = e;
            idx = r.bestv * 8 + e0;
        }
        Z = wave_sum(Z); S2 = wave_sum(S2);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) idx = min(idx, __shfl_xor(idx, o, kWave));
        if ((tid & 63) == 0) { EntPartial e; e.m = gmx; e.Z = Z; e.S = S2; e.idx = idx; e.gs = -INFINITY; e.gidx = 0x7FFFFFFF; s_fin[tid >> 6] = e; }
        __syncthreads();
        if (tid == 0) {
            EntPartial e;
            e.m = gmx > kEntNone ? gmx : -INFINITY;
            e.Z = ((s_fin[0].Z + s_fin[1].Z) + s_fin[2].Z) + s_fin[3].Z;
            e.S = (((s_fin[0].S + s_fin[1].S) + s_fin[2].S) + s_fin[3].S) * kLn2;
            e.idx = min(min(s_fin[0].idx, s_fin[1].idx), min(s_fin[2].idx, s_fin[3].idx));
            e.gs = -INFINITY; e.gidx = 0x7FFFFFFF;          // no sampling on materialised logits
            a.partials[item] = e;
        }
        item = __builtin_amdgcn_readfirstlane(nitem); it = nit;
        return !more;
    };
    // the first-half registers alternate between A and C, so no request ever has to land
    // before the loop can go round
    for (;;) {
        if (one_item(A, C)) break;
        if (one_item(C, A)) break;
    }
}

// ---------------------------------------------------------------------------------------
// The same pass with window and switch rule taken along (small windows): one workgroup takes a whole
// row of one step -- its chunks one after the other, the threads' running statistics carried across
// them, one reduction over the workgroup per row instead of one per chunk and no partials in memory --
// and leaves the row's entropy and arg max.  The workgroup that does so for the last of a row's steps
// in this launch (arrival counter per row, left at zero) reads the row's entropies back and takes its
// window and switch rule through the steps in order.  One launch per up to kGateMaxSteps steps.
// ---------------------------------------------------------------------------------------
constexpr int kGateFoldWindow = 64;     // largest window this kernel serves (its LDS copy of the ring)

template <typename T>
struct EntRowArgs {
    const T *step_logits[kGateMaxSteps];      // one [rows, V] matrix per step of the launch
    int V, rows, steps, chunks, vec_per_item; // a row is walked in `chunks` pieces of vec_per_item vectors (<= 8 per thread)
    float *pair_H;                            // [steps * rows]: the entropies, handed between workgroups (written through)
    int *row_tickets;                         // [rows] arrival counters, zero between launches
    GateStepArgs gate;                        // state, configuration and outputs (partials unused)
};

template <typename T>
__device__ __forceinline__ EntItem<T> ent_row_item(const EntRowArgs<T> &a, int pair, int chunk) {
    const int row = pair % a.rows, z = pair / a.rows;
    EntItem<T> it;
    it.base = a.step_logits[z] + (size_t)row * a.V;
    it.v0 = chunk * a.vec_per_item;
    it.v1 = min(it.v0 + a.vec_per_item, a.V >> 3);
    return it;
}

template <typename T>
__global__ __launch_bounds__(256) void k_entropy_rows(EntRowArgs<T> a) {
    __shared__ float s_max[4], s_Z[4], s_S[4];
    __shared__ int s_idx[4], s_last_row;
    __shared__ float s_H[kGateMaxSteps], s_hb[kGateMaxSteps], s_ring[kGateFoldWindow];
    const int tid = threadIdx.x, pairs = a.steps * a.rows;
    int pair = blockIdx.x, chunk = 0;       // uniform: kept in scalar registers
    if (pair >= pairs) return;
    EntItem<T> it = ent_row_item(a, pair, 0);
    Vec8<T> A[4], B[4], C[4];
    ent_load4(A, it, 0);
    EntRun<T> r; r.m = kEntNone; r.Z = 0.f; r.S2 = 0.f; r.bestv = 0; r.best.zero();
    // one piece of a row: `first` holds its first half (already requested), B takes its second half and
    // `next` the first half of the piece after it (the row's next piece, or the first of this workgroup's
    // next row).  Returns true after the last piece.
    auto one_piece = [&](Vec8<T> (&first)[4], Vec8<T> (&next)[4]) __attribute__((always_inline)) -> bool {
        ent_load4(B, it, 4);
        const bool row_done = chunk + 1 == a.chunks;
        const int npair = row_done ? pair + (int)gridDim.x : pair, nchunk = row_done ? 0 : chunk + 1;
        const bool more = npair < pairs;
        const EntItem<T> nit = ent_row_item(a, more ? npair : pair, more ? nchunk : chunk);
        __builtin_amdgcn_sched_barrier(0);
        ent_take4(first, r, it, 0);
        __builtin_amdgcn_sched_barrier(0);
        ent_load4(next, nit, 0);
        __builtin_amdgcn_sched_barrier(0);
        ent_take4(B, r, it, 4);
        if (row_done) {
            // the row's maximum; every thread moves its sums to that reference once, so the
            // rest of the reduction is plain sums in a fixed order
            const float wmx = wave_max(r.m);
            if ((tid & 63) == 0) s_max[tid >> 6] = wmx;
            __syncthreads();
            const float gmx = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
            const float delta = (gmx - r.m) * kLog2e;
            const float sc = __builtin_amdgcn_exp2f(-fminf(delta, 160.f));
            float S2 = sc * (r.S2 - delta * r.Z), Z = r.Z * sc;
            int idx = 0x7FFFFFFF;
            if (r.m == gmx && r.m > kEntNone) {
                float f[8];
                r.best.unpack(f);
                int e0 = 8;
#pragma unroll
                for (int e = 7; e >= 0; --e) if (f[e] == r.m) e0 = e;
                idx = r.bestv * 8 + e0;
            }
            Z = wave_sum(Z); S2 = wave_sum(S2);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) idx = min(idx, __shfl_xor(idx, o, kWave));
            if ((tid & 63) == 0) { s_Z[tid >> 6] = Z; s_S[tid >> 6] = S2; s_idx[tid >> 6] = idx; }
            __syncthreads();
            const int row = pair % a.rows;
            if (tid == 0) {
                EntStat st; st.init();
                st.m = gmx > kEntNone ? gmx : -INFINITY;
                st.Z = ((s_Z[0] + s_Z[1]) + s_Z[2]) + s_Z[3];
                st.S = (((s_S[0] + s_S[1]) + s_S[2]) + s_S[3]) * kLn2;
                st.idx = min(min(s_idx[0], s_idx[1]), min(s_idx[2], s_idx[3]));
                const float H = entropy_from(st, a.gate.unit);
                if (a.gate.H_out) a.gate.H_out[pair] = H;
                if (a.gate.argmax_out) a.gate.argmax_out[pair] = st.idx;
                // hand the entropy over; the row's last arrival in this launch takes the gate
                st_coherent(a.pair_H + pair, H);
                wait_stores();
                const int t = __hip_atomic_fetch_add(a.row_tickets + row, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_last_row = t == a.steps - 1 ? 1 : 0;
                if (t == a.steps - 1) st_coherent(a.row_tickets + row, 0);
            }
            __syncthreads();
            if (s_last_row) {
                if (tid < a.steps) s_H[tid] = ld_coherent(a.pair_H + (size_t)tid * a.rows + row);
                __syncthreads();
                gate_row_apply(a.gate, row, s_H, s_ring, s_hb);      // ends with a barrier
            }
            r.m = kEntNone; r.Z = 0.f; r.S2 = 0.f; r.bestv = 0; r.best.zero();
        }
        pair = __builtin_amdgcn_readfirstlane(npair); chunk = __builtin_amdgcn_readfirstlane(nchunk); it = nit;
        return !more;
    };
    for (;;) {
        if (one_piece(A, C)) break;
        if (one_piece(C, A)) break;
    }
}

// One workgroup per row, one wave per step of the launch: the waves finish the entropies
// of their steps from the partials side by side; window and switch rule follow (gate_row_apply).
constexpr int kGateMaxWindow = 4096;    // largest rolling window w (entries kept in LDS)

__global__ __launch_bounds__(kGateMaxSteps * 64) void k_gate_step(GateStepArgs a) {
    __shared__ float s_H[kGateMaxSteps], s_hb[kGateMaxSteps];
    __shared__ float s_ring[kGateMaxWindow];
    const int r = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (r >= a.rows) return;
    if (wave < a.steps) {
        const size_t o = (size_t)wave * a.rows + r;
        float H;
        if (a.partials) {
            EntStat st = merge_partials(a.partials + o * a.n_part, a.n_part);
            H = entropy_from(st, a.unit);
            if (lane == 0) {
                if (a.H_out) a.H_out[o] = H;
                if (a.argmax_out) a.argmax_out[o] = st.idx;
            }
        } else {
            H = a.H[o];
        }
        if (lane == 0) s_H[wave] = H;
    }
    __syncthreads();
    if (!a.st.ring) return;
    gate_row_apply(a, r, s_H, s_ring, s_hb);
}

}  // namespace ead
