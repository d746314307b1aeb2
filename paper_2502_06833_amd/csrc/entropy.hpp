// Entropy of the next-token distribution (Eq. 1-2), arg max, rolling window (Eq. 3)
// and the switch rule (Eq. 4 / Algorithm 1's switching block).
#pragma once
#include "common.hpp"
#include "linear.hpp"

namespace ead {

constexpr float kLn2Inv = 1.4426950408889634f;

// H = ln Z - S/Z in nats, or divided by ln 2 for bits
__device__ __forceinline__ float entropy_from(const EntStat &s, int unit) {
    float H = logf(s.Z) - s.S / s.Z;
    return unit ? H * kLn2Inv : H;
}

// ---------------------------------------------------------------------------------------
// Stand-alone pass over a logits matrix [rows, V]: grid (chunks, rows, steps), 256 threads.
// Two bytes per logit leave only a handful of ALU operations per element before the
// kernel stops being bandwidth-bound, so the work per logit is pared down:
//  * each thread takes up to NV vectors of 8 logits, finds their maximum first and only
//    then exponentiates: one rescale per thread, not one per element;
//  * the exponentials are taken in base 2 (the hardware instruction): d = (l - m) log2 e is
//    one FMA, Z = sum 2^d, S2 = sum 2^d d, and S = S2 ln 2 once per thread;
//  * d is clamped at -160, where 2^d is 0 in fp32, so -inf logits need no test;
//  * the arg max index is looked up afterwards, only by the threads that hold the
//    workgroup's maximum.
// ---------------------------------------------------------------------------------------
template <typename T>
struct EntArgs {
    const T *logits; int V; int vec_per_wg;   // 8-element vectors per workgroup
    EntPartial *partials;                     // [steps][rows][gridDim.x]
    const T *const *list; int list_n, list_first;   // optional: step z reads list[(list_first + z) % list_n]
};

constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

template <typename T, int NV>
__global__ __launch_bounds__(256) void k_entropy_partial(EntArgs<T> a) {
    __shared__ EntPartial s_part[4];
    const int row = blockIdx.y, tid = threadIdx.x;
    const T *base = (a.list ? a.list[(a.list_first + blockIdx.z) % a.list_n] : a.logits) + (size_t)row * a.V;
    const int nvec = a.V >> 3;
    const int v0 = blockIdx.x * a.vec_per_wg, v1 = min(v0 + a.vec_per_wg, nvec);
    float f[NV][8];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = v0 + tid + i * 256;
        if (v < v1) {
            Vec8<T> x; x.load_stream(base + (size_t)v * 8); x.unpack(f[i]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[i][e] = -INFINITY;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, f[i][e]);
    }
    EntStat st; st.init();
    if (mx > -INFINITY) {
        const float off = -mx * kLog2e;
        float Z = 0.f, S2 = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = fmaxf(fmaf(f[i][e], kLog2e, off), -160.f);
                const float ex = __builtin_amdgcn_exp2f(d);
                Z += ex;
                S2 = fmaf(ex, d, S2);
            }
        }
        st.m = mx; st.Z = Z; st.S = S2 * kLn2; st.idx = tid;      // idx: provisional, the owner thread
    }
    // the workgroup's maximum; then only its holders look their index up
    const float wmx = wave_max(mx);
    if ((tid & 63) == 0) s_part[tid >> 6].m = wmx;
    __syncthreads();
    const float gmx = fmaxf(fmaxf(s_part[0].m, s_part[1].m), fmaxf(s_part[2].m, s_part[3].m));
    __syncthreads();
    if (mx == gmx && mx > -INFINITY) {
        int idx = 0x7FFFFFFF;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = v0 + tid + i * 256;
#pragma unroll
            for (int e = 0; e < 8; ++e) if (f[i][e] == mx) idx = min(idx, v * 8 + e);
        }
        st.idx = idx;
    } else {
        st.idx = 0x7FFFFFFF;
    }
    st = wave_merge(st);
    if ((tid & 63) == 0) { EntPartial e; e.m = st.m; e.Z = st.Z; e.S = st.S; e.idx = st.idx; s_part[tid >> 6] = e; }
    __syncthreads();
    if (tid == 0) {
        EntStat r; r.init();
        for (int w = 0; w < 4; ++w) { EntStat q; q.m = s_part[w].m; q.Z = s_part[w].Z; q.S = s_part[w].S; q.idx = s_part[w].idx; r.merge(q); }
        // scalar tail of a vocabulary that is not a multiple of 8 (last chunk only)
        if (blockIdx.x == gridDim.x - 1) {
            for (int i = nvec * 8; i < a.V; ++i) {
                EntStat q; q.m = to_f32(base[i]); q.Z = q.m > -INFINITY ? 1.f : 0.f; q.S = 0.f; q.idx = i;
                r.merge(q);
            }
        }
        EntPartial e; e.m = r.m; e.Z = r.Z; e.S = r.S; e.idx = r.idx;
        a.partials[((size_t)blockIdx.z * gridDim.y + row) * gridDim.x + blockIdx.x] = e;
    }
}

// Merge n partials of one row in a fixed order (lane i takes i, i+64, ...; then the
// wave tree).  Every lane returns the merged statistics.
__device__ __forceinline__ EntStat merge_partials(const EntPartial *p, int n) {
    EntStat st; st.init();
    for (int i = threadIdx.x & 63; i < n; i += 64) {
        EntStat q; q.m = p[i].m; q.Z = p[i].Z; q.S = p[i].S; q.idx = p[i].idx;
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

// One workgroup per row, one wave per step of the launch: the waves finish the entropies
// of their steps from the partials side by side, then one thread takes the steps in order
// through the window and the switch rule (which make them sequential per row).
constexpr int kGateMaxSteps = 16;

__global__ __launch_bounds__(kGateMaxSteps * 64) void k_gate_step(GateStepArgs a) {
    __shared__ float s_H[kGateMaxSteps];
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
    if (threadIdx.x == 0 && a.st.ring) {
        int model = a.st.model[r], c = a.st.c[r], n = a.st.n[r];
        for (int s = 0; s < a.steps; ++s) {
            const size_t o = (size_t)s * a.rows + r;
            if (a.model_id_out) a.model_id_out[o] = (uint8_t)model;
            const float hb = gate_update(a.st.ring + (size_t)r * a.cfg.w, n, s_H[s], a.cfg, &model, &c);
            ++n;
            if (a.Hbar_out) a.Hbar_out[o] = hb;
            if (a.next_out) a.next_out[o] = (uint8_t)model;
        }
        a.st.model[r] = model; a.st.c[r] = c; a.st.n[r] = n;
    }
}

}  // namespace ead
