// Grouped-query attention of token rows over the KV cache.
//
// A wave handles one (token row, KV head, key range): it streams that range of K and V
// once and serves all G = n_heads / n_kv_heads query heads that share the KV head.
// hd/8 lanes cover one key (8 elements = one 16-byte load each for bf16), so a wave
// works on 64/(hd/8) keys per iteration, each lane group keeping its own online
// soft-max state; groups are merged at the end, and key ranges (splits) are merged by
// k_attn_combine.  Causality comes from the cache itself: row t reads keys 0..pos_t.
#pragma once
#include "common.hpp"

namespace ead {

template <typename KT>
struct AttnArgs {
    const float *q;            // [T, H*hd]
    const KT *kcache, *vcache; // this layer: [seq][kv_head][max_seq][hd]
    const int *count, *row_seq, *row_pos;
    int n_heads, n_kv_heads, max_seq;
    int chunk;                 // keys per split
    int max_splits;            // grid.x
    float scale;               // 1/sqrt(hd)
    float *part_o;             // [T*H*max_splits][hd]   un-normalised
    float2 *part_ml;           // [T*H*max_splits]       (max, sum)
    float *out;                // [T, H*hd] fp32 (optional)
    bf16_t *out_tiles;         // bf16 tiles (high parts) of [T, H*hd] for an MFMA consumer (optional)
    bf16_t *out_tiles_lo;      //   and low parts
};

constexpr float kNegBig = -1e30f;

template <int HD>
__device__ __forceinline__ void attn_store(float *out, bf16_t *out_tiles, bf16_t *out_tiles_lo, int t, int H,
                                           int col, float r) {
    if (out) out[(size_t)t * H * HD + col] = r;
    if (out_tiles) {
        const int KC = (H * HD) >> 5;
        const size_t off = tile_offset(t >> 4, col >> 5, KC) + (size_t)(((t & 15) + 16 * ((col & 31) >> 3)) * 8 + (col & 7));
        split_bf16(r, out_tiles[off].u, out_tiles_lo[off].u);
    }
}

// Keys are taken in chunks of NI * (64 / LPK): all K and V loads of a chunk are issued
// before any arithmetic, scores of the chunk are formed, one rescale is applied per chunk
// and then the values are accumulated.  A row whose whole context fits one split is
// finished here; otherwise k_attn_combine merges the splits.
template <typename KT, int HD, int G>
__global__ __launch_bounds__(64) void k_attn(AttnArgs<KT> a) {
    constexpr int LPK = HD / 8;        // lanes per key
    constexpr int KPI = 64 / LPK;      // keys per load instruction
    constexpr int NI = 8;              // load instructions per chunk
    const int t = blockIdx.z;
    if (t >= *a.count) return;
    const int kvh = blockIdx.y, split = blockIdx.x;
    const int pos = a.row_pos[t], nkeys = pos + 1;
    const int k0 = split * a.chunk;
    if (k0 >= nkeys) return;
    const int k1 = min(k0 + a.chunk, nkeys);
    const int nsplit = (nkeys + a.chunk - 1) / a.chunk;
    const int lane = threadIdx.x, slot = lane / LPK, dl = lane % LPK;
    const int H = a.n_heads;

    float qv[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float *qp = a.q + (size_t)t * H * HD + (size_t)(kvh * G + g) * HD + dl * 8;
        float4 x0 = *reinterpret_cast<const float4 *>(qp), x1 = *reinterpret_cast<const float4 *>(qp + 4);
        qv[g][0] = x0.x * a.scale; qv[g][1] = x0.y * a.scale; qv[g][2] = x0.z * a.scale; qv[g][3] = x0.w * a.scale;
        qv[g][4] = x1.x * a.scale; qv[g][5] = x1.y * a.scale; qv[g][6] = x1.z * a.scale; qv[g][7] = x1.w * a.scale;
    }
    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegBig; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
    }
    const size_t base = ((size_t)a.row_seq[t] * a.n_kv_heads + kvh) * (size_t)a.max_seq * HD;
    const KT *kb = a.kcache + base + dl * 8, *vb = a.vcache + base + dl * 8;

    for (int c0 = k0; c0 < k1; c0 += NI * KPI) {
        Vec8<KT> kx[NI], vx[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int kk = c0 + i * KPI + slot;
            if (kk < k1) { kx[i].load(kb + (size_t)kk * HD); vx[i].load(vb + (size_t)kk * HD); }
            else { kx[i].zero(); vx[i].zero(); }
        }
        float s[NI][G];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            float kf[8];
            kx[i].unpack(kf);
            const bool valid = c0 + i * KPI + slot < k1;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d += qv[g][e] * kf[e];
#pragma unroll
                for (int off = 1; off < LPK; off <<= 1) d += __shfl_xor(d, off, kWave);
                s[i][g] = valid ? d : kNegBig;
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mc = s[0][g];
#pragma unroll
            for (int i = 1; i < NI; ++i) mc = fmaxf(mc, s[i][g]);
            const float mn = fmaxf(m[g], mc);
            const float corr = __expf(m[g] - mn);
            l[g] *= corr;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[g][e] *= corr;
            m[g] = mn;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const bool valid = c0 + i * KPI + slot < k1;
                const float p = valid ? __expf(s[i][g] - mn) : 0.f;
                l[g] += p; s[i][g] = p;
            }
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            float vf[8];
            vx[i].unpack(vf);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[g][e] += s[i][g] * vf[e];
        }
    }
    // merge the key slots of the wave
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m2 = __shfl_xor(m[g], off, kWave), l2 = __shfl_xor(l[g], off, kWave);
            const float M = fmaxf(m[g], m2);
            const float ca = __expf(m[g] - M), cb = __expf(m2 - M);
            l[g] = l[g] * ca + l2 * cb;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float o2 = __shfl_xor(o[g][e], off, kWave);
                o[g][e] = o[g][e] * ca + o2 * cb;
            }
            m[g] = M;
        }
    }
    if (nsplit == 1) {                     // whole context in one split: finish here
        if (slot == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float r = 1.f / l[g];
#pragma unroll
                for (int e = 0; e < 8; ++e) attn_store<HD>(a.out, a.out_tiles, a.out_tiles_lo, t, H, (kvh * G + g) * HD + dl * 8 + e, o[g][e] * r);
            }
        }
        return;
    }
    if (slot == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const size_t item = ((size_t)t * H + (kvh * G + g)) * a.max_splits + split;
            float *po = a.part_o + item * HD + dl * 8;
            *reinterpret_cast<float4 *>(po) = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
            *reinterpret_cast<float4 *>(po + 4) = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
            if (dl == 0) a.part_ml[item] = make_float2(m[g], l[g]);
        }
    }
}

// One workgroup of HD threads per (head, token row): merge the splits (rows whose context
// fits one split were finished by k_attn itself).
template <typename KT, int HD>
__global__ __launch_bounds__(HD) void k_attn_combine(AttnArgs<KT> a) {
    const int t = blockIdx.y;
    if (t >= *a.count) return;
    const int h = blockIdx.x, d = threadIdx.x, H = a.n_heads;
    const int nsplit = (a.row_pos[t] + a.chunk) / a.chunk;       // ceil((pos+1)/chunk)
    if (nsplit == 1) return;
    const size_t item0 = ((size_t)t * H + h) * a.max_splits;
    float M = kNegBig;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, a.part_ml[item0 + s].x);
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float2 ml = a.part_ml[item0 + s];
        const float c = __expf(ml.x - M);
        L += ml.y * c;
        acc += a.part_o[(item0 + s) * HD + d] * c;
    }
    attn_store<HD>(a.out, a.out_tiles, a.out_tiles_lo, t, H, h * HD + d, acc / L);
}

}  // namespace ead
