// Weight-streaming linear layers: Y[T, N] = X[T, K] * W[N, K]^T with fused prologues
// (RMSNorm) and epilogues (rotary + KV append, residual add, SwiGLU, entropy statistics).
//
// Two kernels share the tiled weight layout and the epilogues:
//   k_linear_valu  plain FMA path for a handful of token rows (and for fp32 weights);
//                  activations stay fp32, staged once per workgroup in LDS.
//   k_linear_mfma  16x16x32 f16 MFMA path for two or more token rows (batched decode,
//                  catch-up chunks, prompt prefill); activations are half-precision tiles.
// In both, a workgroup owns 16-row blocks of W and its waves split K, so a wave reads
// contiguous streams of 1 KB (2-byte) tiles; partial sums meet in LDS and are added in wave
// order, so a row's result does not depend on how many rows are in flight.
#pragma once
#include "common.hpp"

namespace ead {

enum Epilogue { EPI_QKV = 0, EPI_RES = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct EntPartial { float m, Z, S; int idx; float gs; int gidx; };

template <typename WT>
struct LinArgs {
    const WT *W;            // tiled weights, Np x K
    int Np, K;
    const int *count;       // device: number of activation rows this pass
    const int *rowmap;      // optional: activation row r reads x[rowmap[r]] (LM head), else x[r]
    const float *x;         // fp32 activations [*, ldx]        (VALU path)
    int ldx;
    const bf16_t *xp;       // half-precision activation tiles [K/32][ceil(rows/16)][64][8] (MFMA path; the element type only names the width)
    const float *gain;      // RMSNorm gain (VALU path prologue), null = no norm
    float eps;
    // outputs
    float *out;             // RES: residual stream [T, ldo] (+=); SWIGLU: h [T, ldo]; QKV: q [T, ldo]
    int ldo;
    const WT *res_embed;    // RES, optional: the residual is this embedding row instead of out (first layer)
    bf16_t *out_tiles;      // SWIGLU, optional: h as half-precision tiles for the next MFMA layer
    int tbs;                // token blocks of the pass, (count + 15) / 16: the stride of activation tiles (xp, out_tiles) along k
    // QKV
    WT *kcache, *vcache;    // this layer's cache, [seq][kv_head][max_seq][hd]
    WT *vtcache;            // optional second copy of V, transposed in tiles (vt_offset): the matrix-core attention contracts over keys
    const int *row_seq, *row_pos;
    const float2 *rope;     // [max_seq][hd/2] (cos, sin)
    int n_heads, n_kv_heads, hd, max_seq;
    // LOGITS
    EntPartial *partials;   // [rows][gridDim.x]
    float *logits;          // optional dump [rows][Np]
    // LOGITS with sampling: inverse temperature (0 = greedy), generator key, and where to find
    // the sequence of LM row t and its count of generated tokens
    float samp_inv_t; uint32_t samp_k0, samp_k1;
    const int *samp_seq, *samp_ngen;
    // MFMA path with K split over KS workgroups per row-block group
    int tb_base;            // k_linear_mfma_wt with split K, k_sk_merge: first token block of the sweep this launch takes
    int sweeps;             // without split K: > 1 = one workgroup per (row-block group, sweep of 128 rows; k_linear_mfma_gemm: 256)
    int KS;
    float *sk_part;         // [KS][groups][R][NT][256] partial sums
    int *sk_tickets;        // [groups] arrival counters, zero between launches
};

// ------------------------------------------------------------------------------------
// Epilogue for one output element: packed row p of token row t.  Called by 16-lane
// groups whose lanes hold consecutive packed rows, so the rotary / SwiGLU partner is
// the neighbouring lane.
// ------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ void put(T *p, T v, bool coherent) {
    if (coherent) st_coherent(p, v); else *p = v;
}

// What an epilogue reads from memory for one output element.  It is fetched ahead (before
// the k loop of the FMA path, before the reduction of the MFMA path) so that the chain
// position -> rotary table, or the residual, is not waited for between two barriers.
struct EpiPre { float res; float2 cs; int pos, seq; };

// COH: outputs are handed to other workgroups inside the same kernel (fused decode).
template <typename WT, int EPI, bool COH = false>
__device__ __forceinline__ EpiPre epi_prefetch(const LinArgs<WT> &a, int p, int t, bool valid) {
    EpiPre e; e.res = 0.f; e.cs = make_float2(1.f, 0.f); e.pos = 0; e.seq = 0;
    if (!valid) return e;
    if constexpr (EPI == EPI_RES) {
        const float *dst = a.out + (size_t)t * a.ldo + p;
        e.res = a.res_embed ? to_f32(a.res_embed[p]) : (COH ? ld_coherent(dst) : *dst);
    } else if constexpr (EPI == EPI_QKV) {
        e.pos = a.row_pos[t]; e.seq = a.row_seq[t];
        const int hd = a.hd, NQ = a.n_heads * hd, NK = a.n_kv_heads * hd;
        if (p < NQ + NK) {
            const int pp = p < NQ ? p : p - NQ;
            e.cs = a.rope[(size_t)e.pos * (hd >> 1) + ((pp % hd) >> 1)];
        }
    } else if constexpr (EPI == EPI_LOGITS) {
        if (a.samp_inv_t > 0.f) { e.seq = a.samp_seq[t]; e.pos = a.samp_ngen[e.seq]; }
    }
    return e;
}

template <typename WT, int EPI, bool COH = false>
__device__ __forceinline__ void epilogue(const LinArgs<WT> &a, int p, int t, float v, bool valid,
                                         EntStat &st, const EpiPre &pre) {
    if constexpr (EPI == EPI_RES) {
        if (valid) put(a.out + (size_t)t * a.ldo + p, pre.res + v, COH);
    } else if constexpr (EPI == EPI_SWIGLU) {
        float other = __shfl_xor(v, 1, kWave);       // even lane: gate, odd lane: up
        if (valid && !(p & 1)) {
            float h = v / (1.f + __expf(-v)) * other;
            int i = p >> 1;
            if (a.out) put(a.out + (size_t)t * a.ldo + i, h, COH);
            if (a.out_tiles) {
                size_t off = act_tile_offset(t >> 4, i >> 5, a.tbs) + (size_t)(((t & 15) + 16 * ((i & 31) >> 3)) * 8 + (i & 7));
                a.out_tiles[off].u = f32_to_f16_sat(h);
            }
        }
    } else if constexpr (EPI == EPI_QKV) {
        float other = __shfl_xor(v, 1, kWave);
        if (!valid) return;
        const int hd = a.hd, NQ = a.n_heads * hd, NK = a.n_kv_heads * hd;
        const int pos = pre.pos;
        if (p < NQ + NK) {                            // rotary: lanes (2i, 2i+1) hold dims (i, i+hd/2)
            int pp = p < NQ ? p : p - NQ;
            int head = pp / hd, r = pp % hd, i = r >> 1, s = r & 1;
            const float2 cs = pre.cs;
            float res = s ? (other * cs.y + v * cs.x) : (v * cs.x - other * cs.y);
            int dim = i + s * (hd >> 1);
            if (p < NQ) put(a.out + (size_t)t * a.ldo + head * hd + dim, res, COH);
            else {
                size_t o = (((size_t)pre.seq * a.n_kv_heads + head) * a.max_seq + pos) * hd + dim;
                put(a.kcache + o, from_f32<WT>(res), COH);
            }
        } else {
            int pp = p - NQ - NK, head = pp / hd, dim = pp % hd;
            size_t o = (((size_t)pre.seq * a.n_kv_heads + head) * a.max_seq + pos) * hd + dim;
            put(a.vcache + o, from_f32<WT>(v), COH);
            if (a.vtcache) put(a.vtcache + ((size_t)pre.seq * a.n_kv_heads + head) * hd * a.max_seq + vt_offset(dim, pos, a.max_seq), from_f32<WT>(v), COH);
        }
    } else {                                          // EPI_LOGITS: fold the logit into (m, Z, S, argmax)
        if (!valid) return;
        if (a.logits) a.logits[(size_t)t * a.Np + p] = v;
        if (a.samp_inv_t > 0.f) {                     // perturbed score l/T + g; rows come in rising order
            const float sc = fmaf(v, a.samp_inv_t, gumbel_noise(a.samp_k0, a.samp_k1, pre.seq, pre.pos, p));
            if (sc > st.gs) { st.gs = sc; st.gidx = p; }
        }
        if (st.Z == 0.f) { st.m = v; st.Z = 1.f; st.S = 0.f; st.idx = p; }
        else if (v > st.m) {
            float d = st.m - v, e = __expf(d);
            st.S = e * (st.S + d * st.Z); st.Z = st.Z * e + 1.f; st.m = v; st.idx = p;
        } else {
            float d = v - st.m, e = __expf(d);
            st.S += e * d; st.Z += e;
        }
    }
}

// After a workgroup has seen all its row blocks: merge the 16 lanes of each token row
// and store one partial per (row, workgroup).
template <typename WT, bool COH = false>
__device__ __forceinline__ void logits_flush(const LinArgs<WT> &a, int t, bool valid, EntStat st) {
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
        EntStat q;
        q.m = __shfl_xor(st.m, o, kWave); q.Z = __shfl_xor(st.Z, o, kWave);
        q.S = __shfl_xor(st.S, o, kWave); q.idx = __shfl_xor(st.idx, o, kWave);
        q.gs = __shfl_xor(st.gs, o, kWave); q.gidx = __shfl_xor(st.gidx, o, kWave);
        st.merge(q);
    }
    if (valid && (threadIdx.x & 15) == 0) {
        EntPartial *d = a.partials + (size_t)t * gridDim.x + blockIdx.x;
        put(&d->m, st.m, COH); put(&d->Z, st.Z, COH); put(&d->S, st.S, COH); put(&d->idx, st.idx, COH);
        put(&d->gs, st.gs, COH); put(&d->gidx, st.gidx, COH);
    }
}

// ------------------------------------------------------------------------------------
// FMA path.  TC token rows per pass over the weights; NW waves split K.
// dynamic LDS: xs[TC][K] floats, then red[NW][TC][16] floats.
// A wave's tiles are fetched U at a time, one group ahead of the arithmetic, and the
// first group of the next row block (or of the kernel, before the activations are even
// staged) is already in flight while partial sums are being reduced.
// ------------------------------------------------------------------------------------
template <typename WT, int U>
__device__ __forceinline__ void load_group(Vec8<WT> (&w)[U], const WT *wp, int kc, int kc1) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (kc + u < kc1) w[u].load_stream(wp + (size_t)u * 512);
        else w[u].zero();
    }
}

template <typename WT, int TC, int NW, int EPI>
__global__ __launch_bounds__(NW * 64) void k_linear_valu(LinArgs<WT> a) {
    constexpr int U = sizeof(WT) == 2 ? 8 : 4;
    extern __shared__ float smem[];
    const int K = a.K, KC = K >> 5, NB = a.Np >> 4;
    float *xs = smem;
    float *red = smem + (size_t)TC * K;
    __shared__ float s_ss[NW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4;
    const int T = *a.count;
    const int kc0 = (wave * KC) / NW, kc1 = ((wave + 1) * KC) / NW;

    Vec8<WT> cur[U];
    if ((int)blockIdx.x < NB) load_group<WT, U>(cur, a.W + tile_offset(blockIdx.x, kc0, KC) + lane * 8, kc0, kc1);

    for (int t0 = 0; t0 < T; t0 += TC) {
        // ---- stage (and normalise) TC activation rows ----
        for (int tc = 0; tc < TC; ++tc) {
            const int t = t0 + tc;
            float *xr = xs + (size_t)tc * K;
            if (t < T) {
                const float *src = a.x + (size_t)(a.rowmap ? a.rowmap[t] : t) * a.ldx;
                float ss = 0.f;
                for (int k = tid * 4; k < K; k += NW * 64 * 4) {
                    float4 v = *reinterpret_cast<const float4 *>(src + k);
                    *reinterpret_cast<float4 *>(xr + k) = v;
                    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                }
                if (a.gain) {
                    ss = wave_sum(ss);
                    if (lane == 0) s_ss[wave] = ss;
                    __syncthreads();
                    float tot = 0.f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) tot += s_ss[w];
                    const float inv = 1.0f / sqrtf(tot / (float)K + a.eps);
                    for (int k = tid * 4; k < K; k += NW * 64 * 4) {
                        float4 v = *reinterpret_cast<float4 *>(xr + k);
                        float4 gn = *reinterpret_cast<const float4 *>(a.gain + k);
                        v.x *= inv * gn.x; v.y *= inv * gn.y; v.z *= inv * gn.z; v.w *= inv * gn.w;
                        *reinterpret_cast<float4 *>(xr + k) = v;
                    }
                    __syncthreads();
                }
            } else {
                for (int k = tid * 4; k < K; k += NW * 64 * 4)
                    *reinterpret_cast<float4 *>(xr + k) = make_float4(0, 0, 0, 0);
            }
        }
        __syncthreads();

        EntStat st; st.init();
        for (int rb = blockIdx.x; rb < NB; rb += gridDim.x) {
            float acc[TC];
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) acc[tc] = 0.f;
            const WT *wp = a.W + tile_offset(rb, kc0, KC) + lane * 8;
            const float *xq = xs + g * 8;
            // what the epilogue reads is requested now and arrives during the k loop
            const EpiPre pre = epi_prefetch<WT, EPI>(a, rb * 16 + (tid & 15), t0 + (tid >> 4), tid < 16 * TC && t0 + (tid >> 4) < T);
            for (int kc = kc0; kc < kc1; kc += U) {
                // fetch one group ahead: the rest of this row block, else the head of the next
                // one (the next pass over the same block when more token rows follow)
                Vec8<WT> nxt[U];
                if (kc + U < kc1) load_group<WT, U>(nxt, wp + (size_t)U * 512, kc + U, kc1);
                else {
                    int nrb = rb + gridDim.x;
                    if (nrb >= NB && t0 + TC < T) nrb = blockIdx.x;
                    if (nrb < NB) load_group<WT, U>(nxt, a.W + tile_offset(nrb, kc0, KC) + lane * 8, kc0, kc1);
                    else {
#pragma unroll
                        for (int u = 0; u < U; ++u) nxt[u].zero();
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float wf[8];
                    cur[u].unpack_w(wf);
                    const int kk = min(kc + u, kc1 - 1);          // tiles past the end are zero
#pragma unroll
                    for (int tc = 0; tc < TC; ++tc) {
                        const float4 x0 = *reinterpret_cast<const float4 *>(xq + (size_t)tc * K + kk * 32);
                        const float4 x1 = *reinterpret_cast<const float4 *>(xq + (size_t)tc * K + kk * 32 + 4);
                        acc[tc] += wf[0] * x0.x + wf[1] * x0.y + wf[2] * x0.z + wf[3] * x0.w
                                 + wf[4] * x1.x + wf[5] * x1.y + wf[6] * x1.z + wf[7] * x1.w;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) cur[u] = nxt[u];
                wp += (size_t)U * 512;
            }
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) {
                float v = acc[tc];
                v += __shfl_xor(v, 16, kWave);
                v += __shfl_xor(v, 32, kWave);
                if (lane < 16) red[(wave * TC + tc) * 16 + lane] = v;
            }
            __syncthreads();
            if (tid < 16 * TC) {
                const int tc = tid >> 4, j = tid & 15;
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) v += red[(w * TC + tc) * 16 + j];
                epilogue<WT, EPI>(a, rb * 16 + j, t0 + tc, v, t0 + tc < T, st, pre);
            }
            __syncthreads();
        }
        if constexpr (EPI == EPI_LOGITS) {
            if (tid < 16 * TC) logits_flush<WT>(a, t0 + (tid >> 4), t0 + (tid >> 4) < T, st);
        }
    }
}

// ------------------------------------------------------------------------------------
// MFMA path (bf16).  A workgroup of NW waves owns R row blocks of W at a time and NT
// blocks of 16 token rows; its waves split K.  For every k tile a wave fetches R weight
// tiles (the stream from memory) and the NT activation tiles (from cache), so an activation
// tile is fetched once for R weight tiles: with R = 1 the activation fetches alone would
// take most of a compute unit's load-issue cycles at a batch of 32.  Fetches run a ring of
// D k tiles ahead of the matrix cores; the ring slots are register arrays indexed by the
// unrolled loop, so nothing is copied and a wave keeps D * R KB of weights in flight.
// Both operands are IEEE halves (common.hpp): the weights keep their bf16 values exactly, the
// activations are rounded to 11 significant bits (with bf16-rounded activations the logits of a
// full-depth model drift well past their tolerance; a bf16 hi + lo pair, which this path used
// first, costs two products and twice the activation traffic per weight tile).  Every output
// element accumulates its k tiles in ascending order and the waves' sums
// are added in wave order, whatever R, NT and D are: a row's result does not depend
// on how many rows share the pass (NW is fixed per matrix shape).  Matrices with few row
// blocks and a long K are also split along K over KS workgroups per group (SK), whose sums
// meet in memory; KS follows the matrix shape alone and the slabs are added in order.
// ------------------------------------------------------------------------------------
constexpr int kSplitKMax = 8;       // most K slabs per row-block group

template <int NW, int R, int NT, int D, int EPI, bool SK = false>
__global__ __launch_bounds__(NW * 64) void k_linear_mfma(LinArgs<bf16_t> a) {
    constexpr int NE = (NT * 256 + NW * 64 - 1) / (NW * 64);     // epilogue elements per thread and row block
    __shared__ float red[NW][NT][64][4];
    __shared__ int s_ticket;
    const int K = a.K, KC = K >> 5, NB = a.Np >> 4, NG = (NB + R - 1) / R;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform: keeps the k range in scalar registers
    const int T = *a.count;
    const int TB = (T + 15) >> 4;
    if (TB == 0) return;
    // SK: workgroup (g, ks) takes slab ks of K for row-block group g, and TB <= NT
    const int KS = SK ? a.KS : 1;
    const int ks = SK ? (int)blockIdx.x % KS : 0;
    const int slab0 = (ks * KC) / KS, slab1 = ((ks + 1) * KC) / KS;
    const int kc0 = slab0 + (wave * (slab1 - slab0)) / NW, kc1 = slab0 + ((wave + 1) * (slab1 - slab0)) / NW;
    const int nsteps = kc1 - kc0;
    const int c = (tid >> 4) & 15, j = tid & 15;        // this thread's token column and weight row in the epilogue

    for (int tb0 = 0; tb0 < TB; tb0 += NT) {
        EntStat st[NE];
#pragma unroll
        for (int i = 0; i < NE; ++i) st[i].init();
        const bf16_t *xh[NT];
#pragma unroll
        for (int b = 0; b < NT; ++b)         // token blocks past the end repeat the last one; their results are dropped
            xh[b] = a.xp + act_tile_offset(min(tb0 + b, TB - 1), kc0, TB) + lane * 8;
        const int gstep = SK ? NG : (int)gridDim.x;
        for (int g = SK ? (int)blockIdx.x / KS : (int)blockIdx.x; g < NG; g += gstep) {
            f32x4_t acc[R][NT];
            const bf16_t *wp[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int b = 0; b < NT; ++b) acc[r][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                wp[r] = a.W + tile_offset(min(g * R + r, NB - 1), kc0, KC) + lane * 8;
            }
            Vec8<bf16_t> wa[D][R], xa[D][NT];
            // k tile i of the wave's range into ring slot s; past the end the last tile is
            // fetched again (from cache) and not used, so no branch surrounds the loads
            auto issue = [&](int s, int i) __attribute__((always_inline)) {
                const size_t off = (size_t)max(min(i, nsteps - 1), 0) * 512, xoff = off * TB;
#pragma unroll
                for (int r = 0; r < R; ++r) wa[s][r].load_stream(wp[r] + off);
#pragma unroll
                for (int b = 0; b < NT; ++b) xa[s][b].load(xh[b] + xoff);
            };
#pragma unroll
            for (int s = 0; s < D; ++s) {    // in slot order: the waits below count on it
                issue(s, s);
                __builtin_amdgcn_sched_barrier(0);
            }
            for (int i0 = 0; i0 < nsteps; i0 += D) {
#pragma unroll
                for (int s = 0; s < D; ++s) {
                    if (i0 + s < nsteps) {
#pragma unroll
                        for (int r = 0; r < R; ++r) {
#pragma unroll
                            for (int b = 0; b < NT; ++b)
                                acc[r][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                                    __builtin_bit_cast(f16x8_t, wa[s][r].raw), __builtin_bit_cast(f16x8_t, xa[s][b].raw), acc[r][b], 0, 0, 0);
                        }
                    }
                    // the slot is refilled only after its last reader has been issued: moved any
                    // earlier, the refill needs registers of its own and a copy that waits for it
                    __builtin_amdgcn_sched_barrier(0);
                    issue(s, i0 + s + D);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // what the epilogues read is requested for all row blocks at once
            EpiPre pre[R][NE];
            if (!SK) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < NE; ++i) {
                        const int b = (tid + i * NW * 64) >> 8, t = (tb0 + b) * 16 + c, rb = g * R + r;
                        pre[r][i] = epi_prefetch<bf16_t, EPI>(a, rb * 16 + j, t, b < NT && rb < NB && tb0 + b < TB && t < T);
                    }
            }
            // the waves' partial sums meet in LDS, one row block at a time.  D holds weight
            // row j of token column c in lane c + 16*(j/4), register j%4.
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int b = 0; b < NT; ++b)
                    *reinterpret_cast<float4 *>(&red[wave][b][lane][0]) = make_float4(acc[r][b][0], acc[r][b][1], acc[r][b][2], acc[r][b][3]);
                __syncthreads();
                const int rb = g * R + r;
#pragma unroll
                for (int i = 0; i < NE; ++i) {
                    const int b = (tid + i * NW * 64) >> 8;          // uniform within a wave
                    if (b < NT) {
                        float v = 0.f;
#pragma unroll
                        for (int w = 0; w < NW; ++w) v += red[w][b][c + 16 * (j >> 2)][j & 3];
                        const int t = (tb0 + b) * 16 + c;
                        if constexpr (SK)
                            st_coherent(a.sk_part + ((((size_t)ks * NG + g) * R + r) * NT + b) * 256 + (tid & 255), v);
                        else
                            epilogue<bf16_t, EPI>(a, rb * 16 + j, t, v, rb < NB && tb0 + b < TB && t < T, st[i], pre[r][i]);
                    }
                }
                __syncthreads();
            }
            if constexpr (SK) {
                // the slab's sums are written through to memory; the workgroup that arrives last
                // for this group adds the slabs in order and runs the epilogue.  The counter
                // is left at zero for the next launch.
                wait_stores();
                __syncthreads();
                if (tid == 0) s_ticket = __hip_atomic_fetch_add(a.sk_tickets + g, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
                if (s_ticket == KS - 1) {
                    if (tid == 0) st_coherent(a.sk_tickets + g, 0);
                    // all slabs of all the group's elements, and what the epilogues read, are
                    // requested before the first sum
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int i = 0; i < NE; ++i) {
                            const int b = (tid + i * NW * 64) >> 8, t = (tb0 + b) * 16 + c, rb = g * R + r;
                            pre[r][i] = epi_prefetch<bf16_t, EPI>(a, rb * 16 + j, t, b < NT && rb < NB && tb0 + b < TB && t < T);
                        }
                    float pv[R][NE][kSplitKMax];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int i = 0; i < NE; ++i) {
                            const int b = min((tid + i * NW * 64) >> 8, NT - 1);
#pragma unroll
                            for (int q = 0; q < kSplitKMax; ++q)
                                pv[r][i][q] = ld_coherent(a.sk_part + ((((size_t)min(q, KS - 1) * NG + g) * R + r) * NT + b) * 256 + (tid & 255));
                        }
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const int rb = g * R + r;
#pragma unroll
                        for (int i = 0; i < NE; ++i) {
                            const int b = (tid + i * NW * 64) >> 8;
                            if (b < NT) {
                                float v = 0.f;
#pragma unroll
                                for (int q = 0; q < kSplitKMax; ++q) v += q < KS ? pv[r][i][q] : 0.f;
                                const int t = (tb0 + b) * 16 + c;
                                epilogue<bf16_t, EPI>(a, rb * 16 + j, t, v, rb < NB && tb0 + b < TB && t < T, st[i], pre[r][i]);
                            }
                        }
                    }
                }
            }
        }
        if constexpr (EPI == EPI_LOGITS) {
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                const int b = (tid + i * NW * 64) >> 8;
                if (b < NT) {
                    const int t = (tb0 + b) * 16 + c;
                    logits_flush<bf16_t>(a, t, tb0 + b < TB && t < T, st[i]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// MFMA path for passes of more than 64 token rows (catch-up chunks of many rows, prompt
// prefill): 128 token rows per sweep over the weights.  The activation tiles of a k step
// (8 KB for 128 rows) no longer fit a wave's registers next to a fetch ring, and every
// wave needs all of them, so the four waves of a workgroup walk K together: each fetches a
// quarter of the step's activation tiles (ring of DA steps, like its R weight tiles), the
// quarters meet in LDS (two buffers, one barrier per step), and every wave multiplies its own
// 16 R weight rows with all 128 token rows.  No sums cross waves; a wave turns its accumulators
// to the epilogue's (token column, weight row) order through a private 1 KB of LDS.
// Each output element still accumulates its k tiles in ascending order.
// ------------------------------------------------------------------------------------
// One 16 x 16 block of results in the matrix cores' layout (lane L: weight rows 4*(L/16)..+3 of
// token column L%16) -> the epilogue, which wants neighbouring lanes to hold neighbouring weight
// rows of one token column.  s_tw: 1 KB of LDS owned by the calling wave.
template <int EPI>
__device__ __forceinline__ void block_epilogue(const LinArgs<bf16_t> &a, float (*s_tw)[4], int rb, int tb, f32x4_t d,
                                               bool ok, int T, int lane) {
    EntStat st; st.init();            // unused by the epilogues this is built for
    EpiPre pre[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = k * 64 + lane, c = e >> 4, j = e & 15, t = tb * 16 + c;
        pre[k] = epi_prefetch<bf16_t, EPI>(a, rb * 16 + j, t, ok && t < T);
    }
    *reinterpret_cast<float4 *>(&s_tw[lane][0]) = make_float4(d[0], d[1], d[2], d[3]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = k * 64 + lane, c = e >> 4, j = e & 15, t = tb * 16 + c;
        const float v = s_tw[c + 16 * (j >> 2)][j & 3];
        epilogue<bf16_t, EPI>(a, rb * 16 + j, t, v, ok && t < T, st, pre[k]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kWideTok = 8;          // token blocks (of 16 rows) per sweep

// Passes of more than 32 rows: a workgroup takes RG (8; 7 where that fills the compute units better)
// row blocks and 16 NW TPW token rows per sweep; each of its NW waves owns TPW (1 or 2) token blocks
// and all RG row blocks.  NW follows the pass: four waves for up to 64 rows (TPW = 1) and for sweeps of
// 128 (TPW = 2), five to eight waves with one block each for 65-128 rows, so that a pass of 72 rows
// multiplies and fetches five blocks' worth, not eight.  A wave's activation fragments (of its
// blocks) come straight from memory in the matrix cores' operand layout and are never
// shared; the step's RG weight tiles, of which each wave fetches at most two, go through LDS (8 KB read per
// wave and step; sharing the activation tiles instead, with a row-block pair per wave, reads 16 KB
// and is no faster).  SK: workgroup (g, ks) takes slab ks of K for group g (one sweep only: TB <= NW TPW)
// and leaves its sums in memory for k_sk_merge.
template <int DA, int EPI, bool SK = false, int TPW = 2, int RG = 8, int NW = 4>
__global__ __launch_bounds__(NW * 64) void k_linear_mfma_wt(LinArgs<bf16_t> a) {
    static_assert(RG >= 5 && RG <= 8 && NW >= 4 && NW <= 8, "each wave fetches at most two of the workgroup's weight tiles");
    constexpr int NT = NW * TPW;                       // token blocks per sweep (TPW per wave); RG row blocks per workgroup
    constexpr int WPT = (RG + NW - 1) / NW;            // weight tiles a wave fetches per step: tiles wave, wave + NW
    __shared__ __attribute__((aligned(16))) bf16_t s_w[2][8][512];
    __shared__ __attribute__((aligned(16))) float s_t[NW][64][4];
    const int K = a.K, KCfull = K >> 5, NB = a.Np >> 4, NG = (NB + RG - 1) / RG;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T = *a.count;
    const int TB = (T + 15) >> 4;
    if (TB == 0) return;
    const int KS = SK ? a.KS : 1;
    int g = SK ? (int)blockIdx.x / KS : (int)blockIdx.x, tb_first = SK ? a.tb_base : 0;
    const int ks = SK ? (int)blockIdx.x % KS : 0;
    const bool one_sweep = SK || a.sweeps > 1;
    if (!SK && a.sweeps > 1) {
        // workgroup id -> (group, sweep) such that the sweeps of one group run at about the same time on
        // one XCD (id % 8) and find the group's weight tiles in its L2
        const int q = (int)blockIdx.x >> 3, r = (int)blockIdx.x & 7;
        g = (q / a.sweeps) * 8 + r; tb_first = (q % a.sweeps) * NT;
        if (g >= NG || tb_first >= TB) return;
    }
    const int kbase = (ks * KCfull) / KS, KC = ((ks + 1) * KCfull) / KS - kbase;     // this workgroup's k tiles

    for (int tb0 = tb_first; tb0 < TB; tb0 += one_sweep ? TB : NT) {
        f32x4_t acc[RG][TPW];
        const bf16_t *wp[WPT], *bp[TPW];
#pragma unroll
        for (int j = 0; j < RG; ++j)
#pragma unroll
            for (int q = 0; q < TPW; ++q) acc[j][q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < WPT; ++q)      // a wave whose second tile would lie past RG fetches the last tile again and drops it
            wp[q] = a.W + tile_offset(min(g * RG + min(wave + q * NW, RG - 1), NB - 1), kbase, KCfull) + lane * 8;
#pragma unroll
        for (int q = 0; q < TPW; ++q) {
            const int blk = min(tb0 + wave * TPW + q, TB - 1);
            bp[q] = a.xp + act_tile_offset(blk, kbase, TB) + lane * 8;
        }
        Vec8<bf16_t> wa[DA][WPT], ba[DA][TPW];
        auto issue = [&](int s, int i) __attribute__((always_inline)) {
            const size_t off = (size_t)min(i, KC - 1) * 512;
#pragma unroll
            for (int q = 0; q < WPT; ++q) wa[s][q].load_stream(wp[q] + off);
#pragma unroll
            for (int q = 0; q < TPW; ++q) ba[s][q].load(bp[q] + off * TB);
        };
#pragma unroll
        for (int s = 0; s < DA; ++s) {
            issue(s, s);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int i0 = 0; i0 < KC; i0 += DA) {
#pragma unroll
            for (int s = 0; s < DA; ++s) {
                const int i = i0 + s;
                if (i < KC) {                                  // uniform over the workgroup
                    bf16_t (*buf)[512] = s_w[i & 1];
#pragma unroll
                    for (int q = 0; q < WPT; ++q)
                        if (wave + q * NW < RG)                // uniform over the wave
                            *reinterpret_cast<u32x4_t *>(&buf[wave + q * NW][lane * 8]) = wa[s][q].raw;
                    __syncthreads();
                    u32x4_t fw[RG];
#pragma unroll
                    for (int j = 0; j < RG; ++j) fw[j] = *reinterpret_cast<const u32x4_t *>(&buf[j][lane * 8]);
                    __builtin_amdgcn_sched_barrier(0);
                    // neighbouring products go to different accumulators: none waits for another's result
#pragma unroll
                    for (int j = 0; j < RG; ++j)
#pragma unroll
                        for (int q = 0; q < TPW; ++q)
                            acc[j][q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                                __builtin_bit_cast(f16x8_t, fw[j]), __builtin_bit_cast(f16x8_t, ba[s][q].raw), acc[j][q], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                issue(s, i + DA);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (!SK) {
#pragma unroll
            for (int j = 0; j < RG; ++j)
#pragma unroll
                for (int q = 0; q < TPW; ++q) {
                    const int rb = g * RG + j, tb = tb0 + wave * TPW + q;
                    block_epilogue<EPI>(a, s_t[wave], rb, tb, acc[j][q], rb < NB && tb < TB, T, lane);
                }
        } else {
            const size_t slab = (size_t)NG * RG * NT * 256;                // floats per slab
#pragma unroll
            for (int j = 0; j < RG; ++j)
#pragma unroll
                for (int q = 0; q < TPW; ++q) {
                    const int rb = g * RG + j, b = wave * TPW + q;
                    if (rb < NB && tb0 + b < TB) {
                        float *dst = a.sk_part + (size_t)ks * slab + ((size_t)rb * NT + b) * 256 + lane;
                        st_coherent(dst, acc[j][q][0]); st_coherent(dst + 64, acc[j][q][1]);
                        st_coherent(dst + 128, acc[j][q][2]); st_coherent(dst + 192, acc[j][q][3]);
                    }
                }
        }
        __syncthreads();                 // the weight buffers are reused by the next sweep
    }
}

// ------------------------------------------------------------------------------------
// Passes of 33-128 rows, and the 128-row sweeps of longer passes, with the weight stream decoupled from the arithmetic.
// In k_linear_mfma_wt every wave fetches weights (from HBM), fetches activations (from L2) and
// multiplies; a wave's loads complete in order, so its slow weight fetches and its fast
// activation fetches wait for each other, and what a wave can keep in flight is bounded by its
// registers (about 40 KB of weights per compute unit, which at 2-3 us of loaded memory latency
// is 3.5-5 TB/s over the chip).  Here a workgroup has two extra waves that do nothing but fetch
// weight tiles, straight into LDS (the load writes LDS itself: no registers, no ds_write), kDepth - 1
// k steps ahead: up to 104 KB of weights in flight per compute unit.  The NW multiplying waves
// (one token block each, all RG row blocks, as in k_linear_mfma_wt with TPW = 1) fetch only
// their activation fragments, and read a step's weight fragments from LDS while they multiply the step
// before (all waves read all RG tiles: the LDS reads of a step take as long as its products).
// One workgroup barrier per k step hands a step's tiles over; the slot a step leaves is refilled
// right after the next barrier, when every wave has read it.
// The order of the sums of an output element is that of k_linear_mfma_wt.
// ------------------------------------------------------------------------------------
constexpr int kLsDepth = 14;                 // k steps of weight tiles LDS holds (8 KB each)
constexpr int kLsProducers = 2;              // fetching waves; each has 4 (kLsDepth - 1) loads of 1 KB in flight (the counter holds 63)
constexpr size_t kLsLdsBytes(int nw) { return (size_t)kLsDepth * 8 * 1024 + (size_t)nw * 64 * 4 * sizeof(float); }

template <int EPI, bool SK, int NW, int RG>
__global__ __launch_bounds__((NW + kLsProducers) * 64) void k_linear_mfma_ls(LinArgs<bf16_t> a) {
    static_assert(RG >= 5 && RG <= 8 && NW >= 4 && NW <= 8, "a producer wave fetches four of the step's eight tile slots");
    constexpr int DA = 6;                              // ring of activation fragments per multiplying wave
    extern __shared__ __attribute__((aligned(16))) unsigned char ls_smem[];
    bf16_t (*s_w)[8][512] = reinterpret_cast<bf16_t (*)[8][512]>(ls_smem);                       // [kLsDepth][8][512]
    float (*s_t)[64][4] = reinterpret_cast<float (*)[64][4]>(ls_smem + (size_t)kLsDepth * 8 * 1024);   // [NW][64][4]
    const int K = a.K, KCfull = K >> 5, NB = a.Np >> 4, NG = (NB + RG - 1) / RG;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T = *a.count;
    const int TB = (T + 15) >> 4;
    if (TB == 0) return;
    const int KS = SK ? a.KS : 1;
    int g = SK ? (int)blockIdx.x / KS : (int)blockIdx.x, tb0 = SK ? a.tb_base : 0;
    const int ks = SK ? (int)blockIdx.x % KS : 0;
    if (!SK && a.sweeps > 1) {
        // passes of more than 128 rows: one workgroup per (group, 128-row sweep), numbered as in
        // k_linear_mfma_wt so that the sweeps of one group run at about the same time on one XCD
        const int q = (int)blockIdx.x >> 3, r = (int)blockIdx.x & 7;
        g = (q / a.sweeps) * 8 + r; tb0 = (q % a.sweeps) * NW;
        if (g >= NG || tb0 >= TB) return;
    }
    const int kbase = (ks * KCfull) / KS, KC = ((ks + 1) * KCfull) / KS - kbase;     // this workgroup's k tiles
    auto kstep = [&](int j) __attribute__((always_inline)) { return min(j, KC - 1); };      // past the end: the last step again

    if (wave >= NW) {
        // ---- fetching wave p: tile slots p, p + 2, p + 4, p + 6 of every step (slots past RG repeat the last row block) ----
        const int p = wave - NW;
        const bf16_t *wp[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            wp[q] = a.W + tile_offset(min(g * RG + min(p + 2 * q, RG - 1), NB - 1), kbase, KCfull) + lane * 8;
        auto issue = [&](int j) __attribute__((always_inline)) {      // step j (past the end: the last step again, never read)
            const size_t off = (size_t)kstep(j) * 512;
            bf16_t (*slot)[512] = s_w[j % kLsDepth];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wp[q] + off),
                                                 (__attribute__((address_space(3))) void *)&slot[p + 2 * q][0], 16, 0, 0);
        };
        for (int j = 0; j < kLsDepth - 1; ++j) issue(j);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * (kLsDepth - 2)) : "memory");      // step 0 has landed
        __builtin_amdgcn_s_barrier();                 // the bare barrier: this wave has nothing else to wait for
        for (int i = 0; i < KC; ++i) {
            // the multiplying waves read a step's tiles one step ahead of using them: step i + 1 has to
            // have landed; steps i + 2 .. i + kLsDepth - 2 may still be on their way
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * (kLsDepth - 3)) : "memory");
            __builtin_amdgcn_s_barrier();
            issue(i + kLsDepth - 1);                  // into the slot of step i - 1, which every wave has read by now
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // nothing may land in LDS after the workgroup has gone
        return;
    }

    // ---- multiplying wave: token block tb0 + wave, all RG row blocks ----
    f32x4_t acc[RG];
#pragma unroll
    for (int j = 0; j < RG; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int blk = min(tb0 + wave, TB - 1);
    const bf16_t *bp = a.xp + act_tile_offset(blk, kbase, TB) + lane * 8;
    Vec8<bf16_t> ba[DA];
    auto issue = [&](int s, int i) __attribute__((always_inline)) {
        ba[s].load(bp + (size_t)kstep(i) * 512 * TB);
    };
#pragma unroll
    for (int s = 0; s < DA; ++s) {
        issue(s, s);
        __builtin_amdgcn_sched_barrier(0);
    }
    // weight fragments of step i + 1 are read from LDS while step i is multiplied (two register sets)
    static_assert(DA % 2 == 0, "the two fragment sets alternate with the unrolled ring slots");
    u32x4_t fw[2][RG];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < RG; ++j) fw[0][j] = *reinterpret_cast<const u32x4_t *>(&s_w[0][j][lane * 8]);
    for (int i0 = 0; i0 < KC; i0 += DA) {
#pragma unroll
        for (int s = 0; s < DA; ++s) {
            const int i = i0 + s;
            if (i < KC) {                                  // uniform over the workgroup
                __syncthreads();
                bf16_t (*nxt)[512] = s_w[(i + 1) % kLsDepth];      // past the last step: a slot nobody uses
#pragma unroll
                for (int j = 0; j < RG; ++j) fw[(s + 1) & 1][j] = *reinterpret_cast<const u32x4_t *>(&nxt[j][lane * 8]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < RG; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                        __builtin_bit_cast(f16x8_t, fw[s & 1][j]), __builtin_bit_cast(f16x8_t, ba[s].raw), acc[j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue(s, i + DA);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if constexpr (!SK) {
#pragma unroll
        for (int j = 0; j < RG; ++j) {
            const int rb = g * RG + j, tb = tb0 + wave;
            block_epilogue<EPI>(a, s_t[wave], rb, tb, acc[j], rb < NB && tb < TB, T, lane);
        }
    } else {
        const size_t slab = (size_t)NG * RG * NW * 256;                // floats per slab
#pragma unroll
        for (int j = 0; j < RG; ++j) {
            const int rb = g * RG + j, b = wave;
            if (rb < NB && tb0 + b < TB) {
                float *dst = a.sk_part + (size_t)ks * slab + ((size_t)rb * NW + b) * 256 + lane;
                st_coherent(dst, acc[j][0]); st_coherent(dst + 64, acc[j][1]);
                st_coherent(dst + 128, acc[j][2]); st_coherent(dst + 192, acc[j][3]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// Passes of about 500 rows and more (prompt prefill) through a large matrix.  With 128 rows per
// workgroup every wave of k_linear_mfma_ls reads all of a step's weight tiles from LDS for one
// token block: 8 KB of LDS reads per 8 products, which is LDS-bound at half the matrix cores'
// rate, and every workgroup fetches its activation tiles itself.  Here a workgroup covers
// 8 row blocks x 16 token blocks (128 output rows x 256 token rows); its two fetching waves bring
// both the step's 8 weight tiles and its 16 activation tiles into LDS (24 KB per k step,
// kGemmDepth steps), and each of the eight multiplying waves owns 4 row blocks x 4 token blocks:
// 8 KB of LDS reads per 16 products.  Hand-over, slot reuse and the order of the sums of an
// output element (k tiles in ascending order, one accumulator) are those of k_linear_mfma_ls.
// ------------------------------------------------------------------------------------
constexpr int kGemmDepth = 6;                        // k steps of tiles LDS holds
constexpr int kGemmRows = 8, kGemmTok = 16;          // row blocks and token blocks per workgroup
constexpr int kGemmTiles = kGemmRows + kGemmTok;     // 1 KB tiles per k step; each fetching wave brings half of them
constexpr size_t kGemmLdsBytes = (size_t)kGemmDepth * kGemmTiles * 1024 + (size_t)8 * 64 * 4 * sizeof(float);

template <int EPI>
__global__ __launch_bounds__(640) void k_linear_mfma_gemm(LinArgs<bf16_t> a) {
    constexpr int PL = kGemmTiles / 2;                 // loads per fetching wave and k step
    static_assert(PL * (kGemmDepth - 1) <= 63, "the load counter holds 63");
    extern __shared__ __attribute__((aligned(16))) unsigned char ls_smem[];
    bf16_t (*s_w)[kGemmTiles][512] = reinterpret_cast<bf16_t (*)[kGemmTiles][512]>(ls_smem);    // [kGemmDepth]: weight tiles, then activation tiles
    float (*s_t)[64][4] = reinterpret_cast<float (*)[64][4]>(ls_smem + (size_t)kGemmDepth * kGemmTiles * 1024);
    const int KC = a.K >> 5, NB = a.Np >> 4, NG = (NB + kGemmRows - 1) / kGemmRows;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T = *a.count;
    const int TB = (T + 15) >> 4;
    if (TB == 0) return;
    // workgroup id -> (group, sweep): the sweeps of one group run at about the same time on one XCD (id % 8)
    const int q = (int)blockIdx.x >> 3, r = (int)blockIdx.x & 7;
    const int g = (q / a.sweeps) * 8 + r, tb0 = (q % a.sweeps) * kGemmTok;
    if (g >= NG || tb0 >= TB) return;
    auto kstep = [&](int j) __attribute__((always_inline)) { return min(j, KC - 1); };      // past the end: the last step again

    if (wave >= 8) {
        // ---- fetching wave p: weight tiles p, p + 2, .. and activation tiles p, p + 2, .. of every step ----
        const int p = wave - 8;
        const bf16_t *wp[kGemmRows / 2], *xp[kGemmTok / 2];
#pragma unroll
        for (int j = 0; j < kGemmRows / 2; ++j) wp[j] = a.W + tile_offset(min(g * kGemmRows + p + 2 * j, NB - 1), 0, KC) + lane * 8;
#pragma unroll
        for (int j = 0; j < kGemmTok / 2; ++j) xp[j] = a.xp + act_tile_offset(min(tb0 + p + 2 * j, TB - 1), 0, TB) + lane * 8;
        auto issue = [&](int j) __attribute__((always_inline)) {      // step j (past the end: the last step again, never read)
            const size_t woff = (size_t)kstep(j) * 512, xoff = woff * TB;
            bf16_t (*slot)[512] = s_w[j % kGemmDepth];
#pragma unroll
            for (int i = 0; i < kGemmRows / 2; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wp[i] + woff),
                                                 (__attribute__((address_space(3))) void *)&slot[p + 2 * i][0], 16, 0, 0);
#pragma unroll
            for (int i = 0; i < kGemmTok / 2; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(xp[i] + xoff),
                                                 (__attribute__((address_space(3))) void *)&slot[kGemmRows + p + 2 * i][0], 16, 0, 0);
        };
        for (int j = 0; j < kGemmDepth - 1; ++j) issue(j);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PL * (kGemmDepth - 2)) : "memory");      // step 0 has landed
        __builtin_amdgcn_s_barrier();
        for (int i = 0; i < KC; ++i) {
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PL * (kGemmDepth - 3)) : "memory");  // step i + 1 has landed
            __builtin_amdgcn_s_barrier();
            issue(i + kGemmDepth - 1);                // into the slot of step i - 1, which every wave has read by now
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // nothing may land in LDS after the workgroup has gone
        return;
    }

    // ---- multiplying wave: row blocks 4 wr .. + 3 of the group, token blocks 4 wt .. + 3 of the sweep ----
    const int wr = wave & 1, wt = wave >> 1;
    f32x4_t acc[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[j][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    u32x4_t fw[2][4], fx[2][4];                       // fragments of step i + 1 are read while step i is multiplied
    auto fetch = [&](int set, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) fw[set][j] = *reinterpret_cast<const u32x4_t *>(&s_w[slot][4 * wr + j][lane * 8]);
#pragma unroll
        for (int b = 0; b < 4; ++b) fx[set][b] = *reinterpret_cast<const u32x4_t *>(&s_w[slot][kGemmRows + 4 * wt + b][lane * 8]);
    };
    __syncthreads();
    fetch(0, 0);
    for (int i0 = 0; i0 < KC; i0 += 2) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = i0 + s;
            if (i < KC) {                                  // uniform over the workgroup
                __syncthreads();
                fetch((s + 1) & 1, (i + 1) % kGemmDepth);  // past the last step: a slot nobody uses
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[j][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                            __builtin_bit_cast(f16x8_t, fw[s][j]), __builtin_bit_cast(f16x8_t, fx[s][b]), acc[j][b], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int rb = g * kGemmRows + 4 * wr + j, tb = tb0 + 4 * wt + b;
            block_epilogue<EPI>(a, s_t[wave], rb, tb, acc[j][b], rb < NB && tb < TB, T, lane);
        }
}

// Sum of the K slabs that k_linear_mfma_wt<..., SK = true, TPW> left in memory, in slab order, then
// the epilogue.  One wave per 16 x 16 block; grid = ceil(row blocks * NT / 4) workgroups, NT = 4 TPW.
template <int EPI, int NT = kWideTok>
__global__ __launch_bounds__(256) void k_sk_merge(LinArgs<bf16_t> a, int NGR /* row blocks incl. padding */) {
    __shared__ __attribute__((aligned(16))) float s_t[4][64][4];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NB = a.Np >> 4, T = *a.count, TB = (T + 15) >> 4, KS = a.KS;
    const int blk = blockIdx.x * 4 + wave, rb = blk / NT, b = blk % NT;
    if (rb >= NB || a.tb_base + b >= TB) return;
    const size_t slab = (size_t)NGR * NT * 256;
    const float *src = a.sk_part + ((size_t)rb * NT + b) * 256 + lane;
    float pv[kSplitKMax][4];
#pragma unroll
    for (int q = 0; q < kSplitKMax; ++q) {
        const float *sq = src + (size_t)min(q, KS - 1) * slab;
        pv[q][0] = sq[0]; pv[q][1] = sq[64]; pv[q][2] = sq[128]; pv[q][3] = sq[192];
    }
    f32x4_t d = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < kSplitKMax; ++q)
        if (q < KS) { d[0] += pv[q][0]; d[1] += pv[q][1]; d[2] += pv[q][2]; d[3] += pv[q][3]; }
    block_epilogue<EPI>(a, s_t[wave], rb, a.tb_base + b, d, true, T, lane);
}

// ------------------------------------------------------------------------------------
// fp32 activations -> half-precision activation tiles, optionally through RMSNorm.
// One workgroup per token row; rows >= count (padding of the last 16-row block) are zeroed.
// ------------------------------------------------------------------------------------
struct PackArgs {
    const float *x; int ldx;
    const int *count; const int *rowmap;
    const float *gain; float eps;
    bf16_t *out; int K;
};

constexpr int kPackVecs = 15;        // 16-byte pieces of a row per thread: K <= 15 * 4 * 256

__global__ __launch_bounds__(256) void k_pack_act(PackArgs a) {
    __shared__ float s_ss[4];
    const int T = *a.count;
    const int t = blockIdx.x;
    if (t >= ((T + 15) & ~15)) return;
    const int K = a.K, tid = threadIdx.x, TB = (T + 15) >> 4;
    const float *src = t < T ? a.x + (size_t)(a.rowmap ? a.rowmap[t] : t) * a.ldx : nullptr;
    // the row is read once: thread tid keeps elements 4 tid + 1024 i .. + 3, i = 0, 1, ..; the gains are
    // requested with it, so that one round trip to memory covers everything the row needs
    float4 v[kPackVecs], g[kPackVecs];
#pragma unroll
    for (int i = 0; i < kPackVecs; ++i) {
        const int k = tid * 4 + 1024 * i;
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f); g[i] = make_float4(1.f, 1.f, 1.f, 1.f);
        if (k < K) {
            if (src) v[i] = *reinterpret_cast<const float4 *>(src + k);
            if (a.gain) g[i] = *reinterpret_cast<const float4 *>(a.gain + k);
        }
    }
    float inv = 1.f;
    if (a.gain) {
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < kPackVecs; ++i) ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
        ss = wave_sum(ss);
        if ((tid & 63) == 0) s_ss[tid >> 6] = ss;
        __syncthreads();
        inv = 1.0f / sqrtf((s_ss[0] + s_ss[1] + s_ss[2] + s_ss[3]) / (float)K + a.eps);
    }
#pragma unroll
    for (int i = 0; i < kPackVecs; ++i) {
        const int k = tid * 4 + 1024 * i;
        if (k < K) {
            float f[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
            if (a.gain) { f[0] *= inv * g[i].x; f[1] *= inv * g[i].y; f[2] *= inv * g[i].z; f[3] *= inv * g[i].w; }
            // four of the eight elements a lane of the consuming product holds: 8 bytes, side by side with the neighbouring thread's
            const size_t off = act_tile_offset(t >> 4, k >> 5, TB) + (size_t)(((t & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7));
            uint2 r;
            r.x = (uint32_t)f32_to_f16_sat(f[0]) | ((uint32_t)f32_to_f16_sat(f[1]) << 16);
            r.y = (uint32_t)f32_to_f16_sat(f[2]) | ((uint32_t)f32_to_f16_sat(f[3]) << 16);
            *reinterpret_cast<uint2 *>(a.out + off) = r;
        }
    }
}

}  // namespace ead
