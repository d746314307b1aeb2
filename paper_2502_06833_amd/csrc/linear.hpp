// Weight-streaming linear layers: Y[T, N] = X[T, K] * W[N, K]^T with fused prologues
// (RMSNorm) and epilogues (rotary + KV append, residual add, SwiGLU, entropy statistics).
//
// Two kernels share the tiled weight layout and the epilogues:
//   k_linear_valu  plain FMA path for a handful of token rows (and for fp32 weights);
//                  activations stay fp32, staged once per workgroup in LDS.
//   k_linear_mfma  16x16x32 bf16 MFMA path for wider batches of token rows (decode at
//                  batch > 4, catch-up chunks, prompt prefill); activations are bf16 tiles.
// In both, one workgroup owns a 16-row block of W at a time and its waves split K, so a
// wave reads one contiguous stream of 1 KB (bf16) tiles; partial sums meet in LDS and are
// added in wave order, so a row's result does not depend on how many rows are in flight.
#pragma once
#include "common.hpp"

namespace ead {

enum Epilogue { EPI_QKV = 0, EPI_RES = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct EntPartial { float m, Z, S; int idx; };

template <typename WT>
struct LinArgs {
    const WT *W;            // tiled weights, Np x K
    int Np, K;
    const int *count;       // device: number of activation rows this pass
    const int *rowmap;      // optional: activation row r reads x[rowmap[r]] (LM head), else x[r]
    const float *x;         // fp32 activations [*, ldx]        (VALU path)
    int ldx;
    const bf16_t *xp;       // bf16 activation tiles [ceil(rows/16)][K/32][64][8] (MFMA path): high parts
    const bf16_t *xp_lo;    //   and low parts (activation = hi + lo)
    const float *gain;      // RMSNorm gain (VALU path prologue), null = no norm
    float eps;
    // outputs
    float *out;             // RES: residual stream [T, ldo] (+=); SWIGLU: h [T, ldo]; QKV: q [T, ldo]
    int ldo;
    const WT *res_embed;    // RES, optional: the residual is this embedding row instead of out (first layer)
    bf16_t *out_tiles;      // SWIGLU, optional: h as bf16 tiles (high parts) for the next MFMA layer
    bf16_t *out_tiles_lo;   //   and low parts
    int out_KC;             //   K/32 of that consumer
    // QKV
    WT *kcache, *vcache;    // this layer's cache, [seq][kv_head][max_seq][hd]
    const int *row_seq, *row_pos;
    const float2 *rope;     // [max_seq][hd/2] (cos, sin)
    int n_heads, n_kv_heads, hd, max_seq;
    // LOGITS
    EntPartial *partials;   // [rows][gridDim.x]
    float *logits;          // optional dump [rows][Np]
};

// ------------------------------------------------------------------------------------
// Epilogue for one output element: packed row p of token row t.  Called by 16-lane
// groups whose lanes hold consecutive packed rows, so the rotary / SwiGLU partner is
// the neighbouring lane.
// ------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ void put(T *p, T v, bool coherent) {
    if (coherent) st_coherent(p, v); else *p = v;
}

// COH: outputs are handed to other workgroups inside the same kernel (fused decode).
template <typename WT, int EPI, bool COH = false>
__device__ __forceinline__ void epilogue(const LinArgs<WT> &a, int p, int t, float v, bool valid,
                                         EntStat &st) {
    if constexpr (EPI == EPI_RES) {
        if (valid) {
            float *dst = a.out + (size_t)t * a.ldo + p;
            const float r = a.res_embed ? to_f32(a.res_embed[p]) : (COH ? ld_coherent(dst) : *dst);
            put(dst, r + v, COH);
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        float other = __shfl_xor(v, 1, kWave);       // even lane: gate, odd lane: up
        if (valid && !(p & 1)) {
            float h = v / (1.f + __expf(-v)) * other;
            int i = p >> 1;
            if (a.out) put(a.out + (size_t)t * a.ldo + i, h, COH);
            if (a.out_tiles) {
                size_t off = tile_offset(t >> 4, i >> 5, a.out_KC) + (size_t)(((t & 15) + 16 * ((i & 31) >> 3)) * 8 + (i & 7));
                split_bf16(h, a.out_tiles[off].u, a.out_tiles_lo[off].u);
            }
        }
    } else if constexpr (EPI == EPI_QKV) {
        float other = __shfl_xor(v, 1, kWave);
        if (!valid) return;
        const int hd = a.hd, NQ = a.n_heads * hd, NK = a.n_kv_heads * hd;
        const int pos = a.row_pos[t];
        if (p < NQ + NK) {                            // rotary: lanes (2i, 2i+1) hold dims (i, i+hd/2)
            int pp = p < NQ ? p : p - NQ;
            int head = pp / hd, r = pp % hd, i = r >> 1, s = r & 1;
            float2 cs = a.rope[(size_t)pos * (hd >> 1) + i];
            float res = s ? (other * cs.y + v * cs.x) : (v * cs.x - other * cs.y);
            int dim = i + s * (hd >> 1);
            if (p < NQ) put(a.out + (size_t)t * a.ldo + head * hd + dim, res, COH);
            else {
                size_t o = (((size_t)a.row_seq[t] * a.n_kv_heads + head) * a.max_seq + pos) * hd + dim;
                put(a.kcache + o, from_f32<WT>(res), COH);
            }
        } else {
            int pp = p - NQ - NK, head = pp / hd, dim = pp % hd;
            size_t o = (((size_t)a.row_seq[t] * a.n_kv_heads + head) * a.max_seq + pos) * hd + dim;
            put(a.vcache + o, from_f32<WT>(v), COH);
        }
    } else {                                          // EPI_LOGITS: fold the logit into (m, Z, S, argmax)
        if (!valid) return;
        if (a.logits) a.logits[(size_t)t * a.Np + p] = v;
        if (st.Z == 0.f) { st.m = v; st.Z = 1.f; st.S = 0.f; st.idx = p; }
        else if (v > st.m) {
            float d = st.m - v, e = __expf(d);
            st.S = e * (st.S + d * st.Z); st.Z = st.Z * e + 1.f; st.m = v; st.idx = p;
        } else {
            float d = v - st.m, e = __expf(d);
            st.Z += e; st.S += e * d;
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
        st.merge(q);
    }
    if (valid && (threadIdx.x & 15) == 0) {
        EntPartial *d = a.partials + (size_t)t * gridDim.x + blockIdx.x;
        put(&d->m, st.m, COH); put(&d->Z, st.Z, COH); put(&d->S, st.S, COH); put(&d->idx, st.idx, COH);
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
                    cur[u].unpack(wf);
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
                epilogue<WT, EPI>(a, rb * 16 + j, t0 + tc, v, t0 + tc < T, st);
            }
            __syncthreads();
        }
        if constexpr (EPI == EPI_LOGITS) {
            if (tid < 16 * TC) logits_flush<WT>(a, t0 + (tid >> 4), t0 + (tid >> 4) < T, st);
        }
    }
}

// ------------------------------------------------------------------------------------
// MFMA path (bf16).  Token rows are processed 64 at a time (four 16-column blocks of
// the B operand, which is read as ready-made tiles); NW waves split K.  Activations are
// kept as hi + lo bf16 tile pairs (two MFMAs per weight tile): with bf16-rounded
// activations alone the logits of a 32-layer model drift past 2 % of their range, and
// the matrix cores have an order of magnitude of headroom at these widths.
// ------------------------------------------------------------------------------------
constexpr int kMfmaTokBlocks = 4;

template <int NW, int EPI>
__global__ __launch_bounds__(NW * 64) void k_linear_mfma(LinArgs<bf16_t> a) {
    __shared__ float red[NW][kMfmaTokBlocks][64][4];
    const int K = a.K, KC = K >> 5, NB = a.Np >> 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = *a.count;
    const int TB = (T + 15) >> 4;
    const int kc0 = (wave * KC) / NW, kc1 = ((wave + 1) * KC) / NW;

    for (int tb0 = 0; tb0 < TB; tb0 += kMfmaTokBlocks) {
        const int nb = min(kMfmaTokBlocks, TB - tb0);
        EntStat st[(kMfmaTokBlocks * 256) / (NW * 64) > 0 ? (kMfmaTokBlocks * 256) / (NW * 64) : 1];
#pragma unroll
        for (auto &s : st) s.init();
        for (int rb = blockIdx.x; rb < NB; rb += gridDim.x) {
            f32x4_t acc[kMfmaTokBlocks];
#pragma unroll
            for (int b = 0; b < kMfmaTokBlocks; ++b) acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            const bf16_t *wp = a.W + tile_offset(rb, kc0, KC) + lane * 8;
            const bf16_t *xp = a.xp + tile_offset(tb0, kc0, KC) + lane * 8;
            const bf16_t *xl = a.xp_lo + tile_offset(tb0, kc0, KC) + lane * 8;
            const size_t xstride = (size_t)KC * 512;
            int kc = kc0;
            for (; kc + 2 <= kc1; kc += 2) {
                Vec8<bf16_t> w0, w1;
                w0.load_stream(wp); w1.load_stream(wp + 512);
#pragma unroll
                for (int b = 0; b < kMfmaTokBlocks; ++b) {
                    if (b < nb) {
                        Vec8<bf16_t> x0, x1, l0, l1;
                        x0.load(xp + b * xstride); x1.load(xp + b * xstride + 512);
                        l0.load(xl + b * xstride); l1.load(xl + b * xstride + 512);
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w0.raw), __builtin_bit_cast(bf16x8_t, l0.raw), acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w0.raw), __builtin_bit_cast(bf16x8_t, x0.raw), acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w1.raw), __builtin_bit_cast(bf16x8_t, l1.raw), acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w1.raw), __builtin_bit_cast(bf16x8_t, x1.raw), acc[b], 0, 0, 0);
                    }
                }
                wp += 1024; xp += 1024; xl += 1024;
            }
            for (; kc < kc1; ++kc) {
                Vec8<bf16_t> w0; w0.load_stream(wp);
#pragma unroll
                for (int b = 0; b < kMfmaTokBlocks; ++b) {
                    if (b < nb) {
                        Vec8<bf16_t> x0, l0; x0.load(xp + b * xstride); l0.load(xl + b * xstride);
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w0.raw), __builtin_bit_cast(bf16x8_t, l0.raw), acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w0.raw), __builtin_bit_cast(bf16x8_t, x0.raw), acc[b], 0, 0, 0);
                    }
                }
                wp += 512; xp += 512; xl += 512;
            }
#pragma unroll
            for (int b = 0; b < kMfmaTokBlocks; ++b)
                *reinterpret_cast<float4 *>(&red[wave][b][lane][0]) = make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
            __syncthreads();
            // element e -> (token block b, token column c, weight row j); D holds row j of
            // column c in lane c + 16*(j/4), register j%4
            int si = 0;
            for (int e = tid; e < kMfmaTokBlocks * 256; e += NW * 64, ++si) {
                const int b = e >> 8, c = (e >> 4) & 15, j = e & 15;
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) v += red[w][b][c + 16 * (j >> 2)][j & 3];
                const int t = (tb0 + b) * 16 + c;
                epilogue<bf16_t, EPI>(a, rb * 16 + j, t, v, b < nb && t < T, st[si]);
            }
            __syncthreads();
        }
        if constexpr (EPI == EPI_LOGITS) {
            int si = 0;
            for (int e = tid; e < kMfmaTokBlocks * 256; e += NW * 64, ++si) {
                const int b = e >> 8, c = (e >> 4) & 15;
                const int t = (tb0 + b) * 16 + c;
                logits_flush<bf16_t>(a, t, b < nb && t < T, st[si]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// fp32 activations -> bf16 activation tiles, optionally through RMSNorm.
// One workgroup per token row; rows >= count (padding of the last 16-row block) are zeroed.
// ------------------------------------------------------------------------------------
struct PackArgs {
    const float *x; int ldx;
    const int *count; const int *rowmap;
    const float *gain; float eps;
    bf16_t *out, *out_lo; int K;
};

__global__ __launch_bounds__(256) void k_pack_act(PackArgs a) {
    __shared__ float s_ss[4];
    const int T = *a.count;
    const int t = blockIdx.x;
    if (t >= ((T + 15) & ~15)) return;
    const int K = a.K, KC = K >> 5, tid = threadIdx.x;
    float inv = 1.f;
    const float *src = t < T ? a.x + (size_t)(a.rowmap ? a.rowmap[t] : t) * a.ldx : nullptr;
    if (a.gain && src) {
        float ss = 0.f;
        for (int k = tid * 4; k < K; k += 1024) {
            float4 v = *reinterpret_cast<const float4 *>(src + k);
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
        ss = wave_sum(ss);
        if ((tid & 63) == 0) s_ss[tid >> 6] = ss;
        __syncthreads();
        inv = 1.0f / sqrtf((s_ss[0] + s_ss[1] + s_ss[2] + s_ss[3]) / (float)K + a.eps);
    }
    for (int k = tid * 8; k < K; k += 2048) {
        float f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (src) {
            float4 v0 = *reinterpret_cast<const float4 *>(src + k), v1 = *reinterpret_cast<const float4 *>(src + k + 4);
            f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
            if (a.gain) {
                float4 g0 = *reinterpret_cast<const float4 *>(a.gain + k), g1 = *reinterpret_cast<const float4 *>(a.gain + k + 4);
                f[0] *= inv * g0.x; f[1] *= inv * g0.y; f[2] *= inv * g0.z; f[3] *= inv * g0.w;
                f[4] *= inv * g1.x; f[5] *= inv * g1.y; f[6] *= inv * g1.z; f[7] *= inv * g1.w;
            }
        }
        const size_t off = tile_offset(t >> 4, k >> 5, KC) + (size_t)(((t & 15) + 16 * ((k & 31) >> 3)) * 8);
        float hi[8], lo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { hi[e] = bf16_to_f32(f32_to_bf16(f[e])); lo[e] = f[e] - hi[e]; }
        store8<bf16_t>(a.out + off, hi);
        store8<bf16_t>(a.out_lo + off, lo);
    }
}

}  // namespace ead
