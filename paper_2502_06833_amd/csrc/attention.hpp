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
    const KT *vtcache;         // V once more, transposed in tiles per (seq, kv_head) (vt_offset; k_attn_mfma), or null
    const int *count, *row_seq, *row_pos;
    int n_heads, n_kv_heads, max_seq;
    int chunk;                 // keys per split
    int max_splits;            // grid.x
    float scale;               // 1/sqrt(hd)
    float *part_o;             // [T*H*max_splits][hd]   un-normalised
    float2 *part_ml;           // [T*H*max_splits]       (max, sum)
    int *tickets;              // [T*n_heads] arrival counters, zero between launches
    float *out;                // [T, H*hd] fp32 (optional)
    bf16_t *out_tiles;         // half-precision tiles of [T, H*hd] for an MFMA consumer (optional)
    // k_attn_mfma, passes of up to kAttnOrderMax rows: the launch's z index -> row, longest context first.
    // A workgroup's time follows its row's context; workgroups are dispatched in index order, so the long
    // ones start first and the short ones fill in behind them instead of the other way round.
    int use_order;
    unsigned char order[128];
};
constexpr int kAttnOrderMax = 128;

constexpr float kNegBig = -1e30f;

template <int HD>
__device__ __forceinline__ void attn_store(float *out, bf16_t *out_tiles, int t, int H,
                                           int col, float r, int TB) {
    if (out) out[(size_t)t * H * HD + col] = r;
    if (out_tiles) {
        const size_t off = act_tile_offset(t >> 4, col >> 5, TB) + (size_t)(((t & 15) + 16 * ((col & 31) >> 3)) * 8 + (col & 7));
        out_tiles[off].u = f32_to_f16_sat(r);
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
// accumulated.  The waves meet in LDS.  With a single split (short contexts; the host makes a
// split cover 128 keys for steps of one or two rows, else at least 512) the workgroup normalises
// and writes the output.
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
    constexpr int NI = 4;              // load instructions per chunk
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
        if (nsplit == 1) attn_store<HD>(a.out, a.out_tiles, t, H, h * HD + dd, acc / L, (count + 15) >> 4);
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
        attn_store<HD>(a.out, a.out_tiles, t, H, h * HD + dd, acc / L, (count + 15) >> 4);
    }
}

// ------------------------------------------------------------------------------------
// The same attention on the matrix cores, for passes of many rows.  With G query heads per
// KV head the kernel above spends about 5 G arithmetic instructions per byte of K/V and is
// bound by them from G = 4 up; here scores and weighted sums are 16x16x32 products.
//
// A workgroup (kAttnMfmaWaves waves) takes one (group of rows, KV head, key split).  A group is up to
// RQ = 16 / G consecutive rows of one sequence (a catch-up chunk, cut at positions that are
// multiples of RQ): their RQ * G query vectors are the 16 columns of every product, so the
// sequence's K and V are streamed once for all of them.  Row t leads a group unless row
// t - 1 belongs to the same sequence and pos_t is not a multiple of RQ; other rows' workgroups
// exit at once.
//
// Per block of 32 keys a wave forms S^T = K Q^T (keys x columns; A = 16 key rows of K as they
// lie in the cache, B = Q^T, q as a bf16 hi + lo pair) in two tiles whose rows are interleaved
// (tile 0: keys 0-3, 8-11, ..; tile 1: keys 4-7, 12-15, ..): lane group l/16 then holds the
// scores of keys 8 (l/16) .. +7 of its column, which is the B operand layout of the second
// product O^T += V^T P^T (hd x columns; A = 16 rows of the transposed V copy, 8 consecutive
// keys per lane; p as a bf16 hi + lo pair).  Online soft-max per column; columns live in
// lane % 16 in S^T and in O^T alike, so the rescale stays inside the lane.  Waves, then key
// splits, are merged as in k_attn.
// ------------------------------------------------------------------------------------
// Four waves of about 240 registers: two workgroups share a compute unit.  With eight waves (one workgroup
// per unit) a pass of 96 ragged rows took 62 instead of 56.5 us per layer: a wave then gets only two or three
// key blocks at these contexts, too few for its two fetch buffers to overlap anything, and the unit idles while its
// one workgroup merges and stores.
constexpr int kAttnMfmaWaves = 4;

template <int HD, int G>
__global__ __launch_bounds__(kAttnMfmaWaves * 64, 2) void k_attn_mfma(AttnArgs<bf16_t> a) {
    constexpr int RQ = 16 / G;            // rows per group
    constexpr int KC = HD / 32;           // k steps of the score product
    constexpr int HB = HD / 16;           // row tiles of O^T
    __shared__ float s_o[kAttnMfmaWaves][HD / 2][17];     // the waves' sums meet here, one half of hd at a time
    __shared__ float s_m[kAttnMfmaWaves][16], s_l[kAttnMfmaWaves][16];
    __shared__ int s_ticket;
    const int t = a.use_order ? (int)a.order[blockIdx.z] : (int)blockIdx.z, tz = gridDim.z;
    // everything the grouping needs is requested at once (indices clamped to the launch's rows)
    const int count = *a.count, pos = a.row_pos[t], prev = a.row_seq[max(t - 1, 0)];
    int rs[RQ];
#pragma unroll
    for (int i = 0; i < RQ; ++i) rs[i] = a.row_seq[min(t + i, tz - 1)];
    if (t >= count) return;
    const int seq = rs[0];
    if (t > 0 && prev == seq && pos % RQ != 0) return;                     // its group's leader serves this row
    int n = 1;
#pragma unroll
    for (int i = 1; i < RQ; ++i)
        if (n == i && t + i < count && rs[i] == seq && (pos + i) % RQ != 0) n = i + 1;
    const int kvh = blockIdx.y, split = blockIdx.x;
    const int nkeys = pos + n;                                             // keys of the group's last row
    const int k0 = split * a.chunk;
    if (k0 >= nkeys) return;
    const int k1 = min(k0 + a.chunk, nkeys);
    const int nsplit = (nkeys + a.chunk - 1) / a.chunk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 15, lg = lane >> 4;
    const int H = a.n_heads;
    const int cr = col / G, cg = col % G;                                  // the column's row in the group and query head
    const bool col_ok = cr < n;
    const int lim = col_ok ? pos + cr : -1;                                // last key the column may see

    // Q^T fragments: column col, hd elements kc*32 + lg*8 .. +8, scaled, as bf16 hi + lo
    bf16x8_t qh[KC], ql[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
        float f[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (col_ok) {
            const float *qp = a.q + (size_t)(t + cr) * H * HD + (size_t)(kvh * G + cg) * HD + kc * 32 + lg * 8;
            const float4 x0 = *reinterpret_cast<const float4 *>(qp), x1 = *reinterpret_cast<const float4 *>(qp + 4);
            f[0] = x0.x; f[1] = x0.y; f[2] = x0.z; f[3] = x0.w; f[4] = x1.x; f[5] = x1.y; f[6] = x1.z; f[7] = x1.w;
        }
        u32x4_t h4, l4;
        uint32_t hw[8], lw[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { uint16_t hi, lo; split_bf16(f[e] * a.scale, hi, lo); hw[e] = hi; lw[e] = lo; }
        h4 = u32x4_t{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16), hw[4] | (hw[5] << 16), hw[6] | (hw[7] << 16)};
        l4 = u32x4_t{lw[0] | (lw[1] << 16), lw[2] | (lw[3] << 16), lw[4] | (lw[5] << 16), lw[6] | (lw[7] << 16)};
        qh[kc] = __builtin_bit_cast(bf16x8_t, h4); ql[kc] = __builtin_bit_cast(bf16x8_t, l4);
    }

    const size_t base = ((size_t)seq * a.n_kv_heads + kvh) * (size_t)a.max_seq * HD;
    const bf16_t *kbase = a.kcache + base + lg * 8;                        // + key * HD + kc * 32
    const bf16_t *vbase = a.vtcache + base + col * 32 + lg * 8;           // + tile (hb, block) * 512, see vt_offset
    // row r of score tile 0 is key 8 (r / 4) + r % 4 of the block, of tile 1 that key + 4
    const int krow = 8 * (col >> 2) + (col & 3);

    f32x4_t acc[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) acc[hb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m = kNegBig, lsum = 0.f;

    auto request = [&](Vec8<bf16_t> (&kx)[2][KC], Vec8<bf16_t> (&vx)[HB], int kb) __attribute__((always_inline)) {
        // blocks and keys past the end of the split are read from its last block / key and masked
        const int kbc = min(kb, ((k1 - 1 - k0) & ~31) + k0);
#pragma unroll
        for (int ti = 0; ti < 2; ++ti) {
            const int key = min(kbc + krow + 4 * ti, k1 - 1);
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) kx[ti][kc].load(kbase + (size_t)key * HD + kc * 32);
        }
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) vx[hb].load(vbase + ((size_t)hb * (a.max_seq >> 5) + (kbc >> 5)) * 512);
    };
    auto take = [&](const Vec8<bf16_t> (&kx)[2][KC], const Vec8<bf16_t> (&vx)[HB], int kb) __attribute__((always_inline)) {
        f32x4_t s0 = f32x4_t{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx[0][kc].raw), ql[kc], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx[1][kc].raw), ql[kc], s1, 0, 0, 0);
        }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx[0][kc].raw), qh[kc], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx[1][kc].raw), qh[kc], s1, 0, 0, 0);
        }
        // this lane: keys kb + 8 lg + e, e = 0..7 (s0 holds e < 4), of column col
        float sc[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
        bool ok[8];
        float mc = kNegBig;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int key = kb + 8 * lg + e;
            ok[e] = key < k1 && key <= lim;
            sc[e] = ok[e] ? sc[e] : kNegBig;
            mc = fmaxf(mc, sc[e]);
        }
        mc = fmaxf(mc, __shfl_xor(mc, 16, kWave));
        mc = fmaxf(mc, __shfl_xor(mc, 32, kWave));
        const float mn = fmaxf(m, mc);
        const float corr = __expf(m - mn);               // 1 while the column has seen no key
        m = mn;
        float ps = 0.f;
        uint32_t hw[8], lw[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = ok[e] ? __expf(sc[e] - mn) : 0.f;
            ps += p;
            uint16_t hi, lo; split_bf16(p, hi, lo); hw[e] = hi; lw[e] = lo;
        }
        lsum = lsum * corr + ps;
        const bf16x8_t ph = __builtin_bit_cast(bf16x8_t, u32x4_t{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16), hw[4] | (hw[5] << 16), hw[6] | (hw[7] << 16)});
        const bf16x8_t pl = __builtin_bit_cast(bf16x8_t, u32x4_t{lw[0] | (lw[1] << 16), lw[2] | (lw[3] << 16), lw[4] | (lw[5] << 16), lw[6] | (lw[7] << 16)});
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            acc[hb][0] *= corr; acc[hb][1] *= corr; acc[hb][2] *= corr; acc[hb][3] *= corr;
        }
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) acc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vx[hb].raw), pl, acc[hb], 0, 0, 0);
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) acc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vx[hb].raw), ph, acc[hb], 0, 0, 0);
    };
    {
        Vec8<bf16_t> ka[2][KC], va[HB], kb2[2][KC], vb2[HB];
        constexpr int STEP = kAttnMfmaWaves * 32;
        int kb = k0 + wave * 32;
        request(ka, va, kb);
        while (kb < k1) {
            request(kb2, vb2, kb + STEP);
            __builtin_amdgcn_sched_barrier(0);
            take(ka, va, kb);
            kb += STEP;
            if (kb >= k1) break;
            request(ka, va, kb + STEP);
            __builtin_amdgcn_sched_barrier(0);
            take(kb2, vb2, kb);
            kb += STEP;
        }
    }
    // the column's sum over the four lane groups (m is already the same in all of them)
    lsum += __shfl_xor(lsum, 16, kWave);
    lsum += __shfl_xor(lsum, 32, kWave);
    // the waves meet in LDS.  acc[hb][j]: hd = hb*16 + 4*lg + j, column col
    if (lg == 0) { s_m[wave][col] = m; s_l[wave][col] = lsum; }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if (half) __syncthreads();
#pragma unroll
        for (int hb = 0; hb < HB / 2; ++hb)
#pragma unroll
            for (int j = 0; j < 4; ++j) s_o[wave][hb * 16 + 4 * lg + j][col] = acc[half * (HB / 2) + hb][j];
        __syncthreads();
        for (int e = tid; e < n * G * (HD / 2); e += kAttnMfmaWaves * 64) {
            const int c = e / (HD / 2), dl = e % (HD / 2), dd = half * (HD / 2) + dl;    // column (row in group * G + head), hd element
            float M = kNegBig;
#pragma unroll
            for (int w = 0; w < kAttnMfmaWaves; ++w) M = fmaxf(M, s_m[w][c]);
            float L = 0.f, o = 0.f;
#pragma unroll
            for (int w = 0; w < kAttnMfmaWaves; ++w) {
                const float cw = __expf(s_m[w][c] - M);
                L += s_l[w][c] * cw;
                o += s_o[w][dl][c] * cw;
            }
            const int tr = t + c / G, h = kvh * G + c % G;
            if (nsplit == 1) attn_store<HD>(a.out, a.out_tiles, tr, H, h * HD + dd, o / L, (count + 15) >> 4);
            else {
                const size_t item = ((size_t)tr * H + h) * a.max_splits + split;
                st_coherent(a.part_o + item * HD + dd, o);
                if (dd == 0) {
                    float *ml = reinterpret_cast<float *>(a.part_ml + item);
                    st_coherent(ml, M); st_coherent(ml + 1, L);
                }
            }
        }
    }
    if (nsplit == 1) return;
    wait_stores();
    __syncthreads();
    int *tk = a.tickets + t * a.n_kv_heads + kvh;
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(tk, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != nsplit - 1) return;
    if (tid == 0) st_coherent(tk, 0);
    for (int e = tid; e < n * G * HD; e += kAttnMfmaWaves * 64) {
        const int c = e / HD, dd = e % HD, tr = t + c / G, h = kvh * G + c % G;
        const size_t item0 = ((size_t)tr * H + h) * a.max_splits;
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
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) {
            const float cw = __expf(mm[sp] - M);
            L += ll[sp] * cw;
            o += oo[sp] * cw;
        }
        attn_store<HD>(a.out, a.out_tiles, tr, H, h * HD + dd, o / L, (count + 15) >> 4);
    }
}


}  // namespace ead
