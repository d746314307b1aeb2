// Grouped-query attention of token rows over the KV cache.
//
// A wave handles one (token row, head group, key range): it streams that range of K and V
// once and serves the group's query heads (all G = n_heads / n_kv_heads heads that share
// the KV head, or a single one).  hd/8 lanes cover one key (8 elements = one 16-byte load each for bf16), so a wave
// works on 64/(hd/8) keys per iteration, each lane group keeping its own online
// soft-max state; groups are merged at the end, and key ranges (splits) are merged by
// whichever split finishes last.  Causality comes from the cache itself: row t reads keys
// 0..pos_t.
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
    int *tickets;              // [T*n_heads] arrival counters, zero between launches
    float *out;                // [T, H*hd] fp32 (optional)
    bf16_t *out_tiles;         // bf16 tiles (high parts) of [T, H*hd] for an MFMA consumer (optional)
    bf16_t *out_tiles_lo;      //   and low parts
};

constexpr float kNegBig = -1e30f;

template <int HD>
__device__ __forceinline__ void attn_store(float *out, bf16_t *out_tiles, bf16_t *out_tiles_lo, int t, int H,
                                           int col, float r, int TB) {
    if (out) out[(size_t)t * H * HD + col] = r;
    if (out_tiles) {
        const size_t off = act_tile_offset(t >> 4, col >> 5, TB) + (size_t)(((t & 15) + 16 * ((col & 31) >> 3)) * 8 + (col & 7));
        split_bf16(r, out_tiles[off].u, out_tiles_lo[off].u);
    }
}

// A workgroup of kAttnWaves waves handles one (token row, group of GW query heads, key split).
// GW = G serves all query heads of a KV head from one pass over its keys (the layout for
// many rows or long contexts, where K/V traffic matters); GW = 1 gives every query head a
// workgroup of its own and re-reads K/V from cache, which is what a decode step of one or a
// few rows wants: it is bound by latency and needs the lanes.
//
// The waves take the split's keys in chunks of NI * (64 / LPK).  Two register sets
// alternate: the next chunk's K and V are requested before the current one is worked on.
// Scores of a chunk are formed, one rescale is applied per chunk and then the values are
// accumulated.  The waves meet in LDS.  With a single split (the usual case: the host makes
// a split cover at least 512 keys) the workgroup normalises and writes the output.
// Otherwise it leaves an un-normalised partial, written through to memory (st_coherent),
// and the workgroup that arrives last (ticket counter per (row, head group)) merges the
// partials with coherent loads, so neither a second launch nor a cache write-back /
// invalidate is needed -- only completion of the stores before the ticket is taken.  The
// counter is left at zero for the next launch.
constexpr int kAttnWaves = 8;
constexpr int kAttnMaxSplits = 16;

template <typename KT, int HD, int G, int GW>
__global__ __launch_bounds__(kAttnWaves * 64) void k_attn(AttnArgs<KT> a) {
    static_assert(GW == G || GW == 1, "a workgroup takes all query heads of a KV head, or one");
    constexpr int LPK = HD / 8;        // lanes per key
    constexpr int KPI = 64 / LPK;      // keys per load instruction
    constexpr int NI = (GW == 1 && sizeof(KT) == 2) ? 8 : 4;   // load instructions per chunk
    constexpr int CH = NI * KPI;
    __shared__ float s_o[kAttnWaves][GW][HD];
    __shared__ float s_m[kAttnWaves][GW], s_l[kAttnWaves][GW];
    __shared__ int s_ticket;
    const int t = blockIdx.z;
    // the three scalars are requested together, before the first of them is needed
    const int count = *a.count, pos = a.row_pos[t], seq = a.row_seq[t];
    if (t >= count) return;
    const int hg = blockIdx.y, split = blockIdx.x;
    const int h0 = hg * GW, kvh = h0 / G;
    const int nkeys = pos + 1;
    const int k0 = split * a.chunk;
    if (k0 >= nkeys) return;
    const int k1 = min(k0 + a.chunk, nkeys);
    const int nsplit = (nkeys + a.chunk - 1) / a.chunk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, slot = lane / LPK, dl = lane % LPK;
    const int H = a.n_heads;

    float qv[GW][8];
#pragma unroll
    for (int g = 0; g < GW; ++g) {
        const float *qp = a.q + (size_t)t * H * HD + (size_t)(h0 + g) * HD + dl * 8;
        float4 x0 = *reinterpret_cast<const float4 *>(qp), x1 = *reinterpret_cast<const float4 *>(qp + 4);
        qv[g][0] = x0.x * a.scale; qv[g][1] = x0.y * a.scale; qv[g][2] = x0.z * a.scale; qv[g][3] = x0.w * a.scale;
        qv[g][4] = x1.x * a.scale; qv[g][5] = x1.y * a.scale; qv[g][6] = x1.z * a.scale; qv[g][7] = x1.w * a.scale;
    }
    float m[GW], l[GW], o[GW][8];
#pragma unroll
    for (int g = 0; g < GW; ++g) {
        m[g] = kNegBig; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
    }
    const size_t base = ((size_t)seq * a.n_kv_heads + kvh) * (size_t)a.max_seq * HD;
    const KT *kb = a.kcache + base + dl * 8, *vb = a.vcache + base + dl * 8;

    // keys past the end of the split are read from its last key and masked in the scores:
    // no branch surrounds the loads
    auto request = [&](Vec8<KT> (&kx)[NI], Vec8<KT> (&vx)[NI], int c0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int kk = min(c0 + i * KPI + slot, k1 - 1);
            kx[i].load(kb + (size_t)kk * HD); vx[i].load(vb + (size_t)kk * HD);
        }
    };
    auto take = [&](const Vec8<KT> (&kx)[NI], const Vec8<KT> (&vx)[NI], int c0) __attribute__((always_inline)) {
        float s[NI][GW];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            float kf[8];
            kx[i].unpack(kf);
            const bool valid = c0 + i * KPI + slot < k1;
#pragma unroll
            for (int g = 0; g < GW; ++g) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d += qv[g][e] * kf[e];
#pragma unroll
                for (int off = 1; off < LPK; off <<= 1) d += __shfl_xor(d, off, kWave);
                s[i][g] = valid ? d : kNegBig;
            }
        }
#pragma unroll
        for (int g = 0; g < GW; ++g) {
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
            for (int g = 0; g < GW; ++g)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[g][e] += s[i][g] * vf[e];
        }
    };
    {
        Vec8<KT> ka[NI], va[NI], kb2[NI], vb2[NI];
        constexpr int STEP = kAttnWaves * CH;
        int c0 = k0 + wave * CH;
        request(ka, va, c0);
        while (c0 < k1) {
            request(kb2, vb2, c0 + STEP);
            __builtin_amdgcn_sched_barrier(0);
            take(ka, va, c0);
            c0 += STEP;
            if (c0 >= k1) break;
            request(ka, va, c0 + STEP);
            __builtin_amdgcn_sched_barrier(0);
            take(kb2, vb2, c0);
            c0 += STEP;
        }
    }
    // merge the key slots of the wave
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < GW; ++g) {
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
    // the waves meet in LDS
    if (slot == 0) {
#pragma unroll
        for (int g = 0; g < GW; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_o[wave][g][dl * 8 + e] = o[g][e];
            if (dl == 0) { s_m[wave][g] = m[g]; s_l[wave][g] = l[g]; }
        }
    }
    __syncthreads();
    for (int e = tid; e < GW * HD; e += kAttnWaves * 64) {
        const int g = e / HD, dd = e % HD;
        float M = kNegBig;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, s_m[w][g]);
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            const float c = __expf(s_m[w][g] - M);
            L += s_l[w][g] * c;
            acc += s_o[w][g][dd] * c;
        }
        const int h = h0 + g;
        if (nsplit == 1) attn_store<HD>(a.out, a.out_tiles, a.out_tiles_lo, t, H, h * HD + dd, acc / L, (count + 15) >> 4);
        else {
            const size_t item = ((size_t)t * H + h) * a.max_splits + split;
            st_coherent(a.part_o + item * HD + dd, acc);
            if (dd == 0) {
                float *ml = reinterpret_cast<float *>(a.part_ml + item);
                st_coherent(ml, M); st_coherent(ml + 1, L);
            }
        }
    }
    if (nsplit == 1) return;
    wait_stores();
    __syncthreads();
    int *tk = a.tickets + t * (H / GW) + hg;
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(tk, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != nsplit - 1) return;
    if (tid == 0) st_coherent(tk, 0);
    for (int e = tid; e < GW * HD; e += kAttnWaves * 64) {
        const int g = e / HD, dd = e % HD, h = h0 + g;
        const size_t item0 = ((size_t)t * H + h) * a.max_splits;
        float mm[kAttnMaxSplits], ll[kAttnMaxSplits], oo[kAttnMaxSplits];
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) {
            if (sp < nsplit) {
                const float *ml = reinterpret_cast<const float *>(a.part_ml + item0 + sp);
                mm[sp] = ld_coherent(ml); ll[sp] = ld_coherent(ml + 1);
                oo[sp] = ld_coherent(a.part_o + (item0 + sp) * HD + dd);
            } else { mm[sp] = kNegBig; ll[sp] = 0.f; oo[sp] = 0.f; }
        }
        float M = kNegBig;
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) M = fmaxf(M, mm[sp]);
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) {
            const float c = __expf(mm[sp] - M);
            L += ll[sp] * c;
            acc += oo[sp] * c;
        }
        attn_store<HD>(a.out, a.out_tiles, a.out_tiles_lo, t, H, h * HD + dd, acc / L, (count + 15) >> 4);
    }
}

}  // namespace ead
