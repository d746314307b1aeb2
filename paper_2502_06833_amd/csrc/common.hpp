// Shared device helpers: storage types, 8-element tile loads, wave64 reductions,
// and the tiled weight layout every linear kernel streams.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ead {

constexpr int kWave = 64;
constexpr int kTileRows = 16;   // weight rows per tile (the M of a 16x16x32 MFMA)
constexpr int kTileK = 32;      // contraction elements per tile
constexpr int kLaneElems = 8;   // elements one lane holds of a tile

struct bf16_t { uint16_t u; };

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4e_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
// round-to-nearest-even; finite inputs and infinities
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v.u); }
template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { bf16_t r; r.u = f32_to_bf16(f); return r; }

// x = hi + lo with both parts bf16: the attention kernels keep their query and probability
// operands this way (about 16 significant bits through the bf16 matrix cores, whose other operand
// is the bf16 K/V cache as it lies in memory).
__device__ __forceinline__ void split_bf16(float f, uint16_t &hi, uint16_t &lo) {
    hi = f32_to_bf16(f);
    lo = f32_to_bf16(f - bf16_to_f32(hi));
}

// ---- IEEE half: the storage format of the linear layers' matrix-core operands ----------------
// The weights of a bf16 model are re-encoded as IEEE half when they are tiled: a bf16 value has 8
// significant bits and half has 11, so every weight of magnitude 2^-24 .. 65504 keeps its value
// bit for bit (smaller ones, far below anything a trained or randomly initialised matrix relies
// on, round to a multiple of 2^-24).  The activations of the matrix-core kernels are rounded
// to half as well (relative error 2^-12, eight times finer than bf16), so one f16 product per
// weight tile replaces the two a bf16 hi + lo activation pair needs.  Half tops out at 65504:
// activation values beyond that saturate instead of turning infinite.
__device__ __forceinline__ uint16_t f32_to_f16_sat(float f) {
    const _Float16 h = (_Float16)fminf(fmaxf(f, -65504.f), 65504.f);
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float f16_to_f32(uint16_t u) { return (float)__builtin_bit_cast(_Float16, u); }

template <typename V> using gptr = const V __attribute__((address_space(1))) *;

// Eight consecutive elements of type T held by one lane.
template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    u32x4_t raw;
    // all sources are device-global memory: say so, or pointers that went through LDS or
    // a struct become flat loads
    __device__ __forceinline__ void load(const bf16_t *p) { raw = *(gptr<u32x4_t>)p; }
    __device__ __forceinline__ void load_stream(const bf16_t *p) { raw = __builtin_nontemporal_load((gptr<u32x4_t>)p); }
    __device__ __forceinline__ void unpack(float (&f)[8]) const {
        f[0] = __uint_as_float(raw.x << 16); f[1] = __uint_as_float(raw.x & 0xFFFF0000u);
        f[2] = __uint_as_float(raw.y << 16); f[3] = __uint_as_float(raw.y & 0xFFFF0000u);
        f[4] = __uint_as_float(raw.z << 16); f[5] = __uint_as_float(raw.z & 0xFFFF0000u);
        f[6] = __uint_as_float(raw.w << 16); f[7] = __uint_as_float(raw.w & 0xFFFF0000u);
    }
    // the same 16 bytes read as eight halves: weight tiles of a bf16 model (see above)
    __device__ __forceinline__ void unpack_w(float (&f)[8]) const {
        // element by element through scalars: a bit cast of raw.y taken as a vector element came out as raw.x
        const uint32_t w0 = raw.x, w1 = raw.y, w2 = raw.z, w3 = raw.w;
        f[0] = f16_to_f32((uint16_t)w0); f[1] = f16_to_f32((uint16_t)(w0 >> 16));
        f[2] = f16_to_f32((uint16_t)w1); f[3] = f16_to_f32((uint16_t)(w1 >> 16));
        f[4] = f16_to_f32((uint16_t)w2); f[5] = f16_to_f32((uint16_t)(w2 >> 16));
        f[6] = f16_to_f32((uint16_t)w3); f[7] = f16_to_f32((uint16_t)(w3 >> 16));
        // keep the conversions as conversions: folded into mixed-precision multiply-adds the FMA kernels ran 4 % slower
#pragma unroll
        for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(f[e]));
    }
    __device__ __forceinline__ void zero() { raw = u32x4_t{0u, 0u, 0u, 0u}; }
};
template <> struct Vec8<float> {
    f32x4e_t lo, hi;
    __device__ __forceinline__ void load(const float *p) { lo = *(gptr<f32x4e_t>)p; hi = *(gptr<f32x4e_t>)(p + 4); }
    __device__ __forceinline__ void load_stream(const float *p) {
        lo = __builtin_nontemporal_load((gptr<f32x4e_t>)p);
        hi = __builtin_nontemporal_load((gptr<f32x4e_t>)(p + 4));
    }
    __device__ __forceinline__ void unpack(float (&f)[8]) const {
        f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w; f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
    }
    __device__ __forceinline__ void unpack_w(float (&f)[8]) const { unpack(f); }      // float weights are stored as they are
    __device__ __forceinline__ void zero() { lo = f32x4e_t{0.f, 0.f, 0.f, 0.f}; hi = lo; }
};

template <typename T> __device__ __forceinline__ void store8(T *p, const float (&f)[8]);
template <> __device__ __forceinline__ void store8<float>(float *p, const float (&f)[8]) {
    *reinterpret_cast<float4 *>(p) = make_float4(f[0], f[1], f[2], f[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
}
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t *p, const float (&f)[8]) {
    uint4 r;
    r.x = (uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16);
    r.y = (uint32_t)f32_to_bf16(f[2]) | ((uint32_t)f32_to_bf16(f[3]) << 16);
    r.z = (uint32_t)f32_to_bf16(f[4]) | ((uint32_t)f32_to_bf16(f[5]) << 16);
    r.w = (uint32_t)f32_to_bf16(f[6]) | ((uint32_t)f32_to_bf16(f[7]) << 16);
    *reinterpret_cast<uint4 *>(p) = r;
}

// eight values as halves (weight tiles of a bf16 model, activation tiles); float weights stay float
__device__ __forceinline__ void store8_half(bf16_t *p, const float (&f)[8]) {
    uint4 r;
    r.x = (uint32_t)f32_to_f16_sat(f[0]) | ((uint32_t)f32_to_f16_sat(f[1]) << 16);
    r.y = (uint32_t)f32_to_f16_sat(f[2]) | ((uint32_t)f32_to_f16_sat(f[3]) << 16);
    r.z = (uint32_t)f32_to_f16_sat(f[4]) | ((uint32_t)f32_to_f16_sat(f[5]) << 16);
    r.w = (uint32_t)f32_to_f16_sat(f[6]) | ((uint32_t)f32_to_f16_sat(f[7]) << 16);
    *reinterpret_cast<uint4 *>(p) = r;
}
__device__ __forceinline__ void store8_w(float *p, const float (&f)[8]) { store8<float>(p, f); }
__device__ __forceinline__ void store8_w(bf16_t *p, const float (&f)[8]) { store8_half(p, f); }

// ---- device-coherent scalar accesses -----------------------------------------------------
// Relaxed agent-scope atomics: the store is written through to memory and the load is
// served coherently across the chip's L2 slices, so data handed between workgroups inside
// one kernel needs no cache write-back / invalidate, only completion of the stores
// (wait_stores) before the hand-over is signalled.
__device__ __forceinline__ float ld_coherent(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_coherent(const int *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coherent(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coherent(int *p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coherent(bf16_t *p, bf16_t v) {
    __hip_atomic_store(&p->u, v.u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- wave64 reductions -------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// ---- tiled weight layout -------------------------------------------------------------
// A matrix with Np rows (multiple of 16) and K columns (multiple of 32) is stored as
// tiles of 16 rows x 32 columns.  Tile (rb, kc) occupies 512 consecutive elements at
// (rb * K/32 + kc) * 512; inside it, lane l of a wave owns the 8 elements
//   row rb*16 + (l & 15), columns kc*32 + (l >> 4)*8 .. +8
// at offset l*8 (2-byte elements are IEEE halves, see above).  This is the register layout of the A operand of the 16x16x32 MFMA,
// so a wave reads a whole row block as one contiguous, fully coalesced stream whether
// it feeds the matrix cores or plain FMAs.
__host__ __device__ __forceinline__ size_t tile_offset(int rb, int kc, int KC) {
    return ((size_t)rb * (size_t)KC + (size_t)kc) * 512;
}
// Activation tiles (16 token rows x 32 columns, same inner layout, the B operand) are ordered
// the other way round: tile (tb, kc) of a pass with TB token blocks sits at (kc * TB + tb) * 512.
// Every workgroup of a linear kernel reads the same TB tiles in the same k step; side by side
// they spread over the memory channels, whereas K/32 tiles apart they fall on one or two.
__host__ __device__ __forceinline__ size_t act_tile_offset(int tb, int kc, int TB) {
    return ((size_t)kc * (size_t)TB + (size_t)tb) * 512;
}

// Transposed copy of V for the matrix-core attention, per (sequence, KV head): tiles of 16 hd
// rows x 32 positions, 1 KB each, ordered [hd / 16][pos / 32]; inside a tile [hd % 16][pos % 32].
// A tile is the A operand of the 16x16x32 product that contracts over keys, read by one
// contiguous 1 KB load.  max_seq is a multiple of 32.
__host__ __device__ __forceinline__ size_t vt_offset(int dim, int pos, int max_seq) {
    return (((size_t)(dim >> 4) * (size_t)(max_seq >> 5) + (size_t)(pos >> 5)) * 16 + (size_t)(dim & 15)) * 32 + (size_t)(pos & 31);
}

// ---- online soft-max statistics for the entropy (Eq. 1-2) ------------------------------
// For a set of logits: m = max, Z = sum exp(l-m), S = sum exp(l-m)(l-m), plus the arg max
// (lowest index on ties).  H = ln Z - S/Z.  merge() combines two disjoint sets.
struct EntStat {
    float m, Z, S;
    int idx;
    // sampling (Algorithm 1's y ~ softmax(l / T)): running maximum of the perturbed scores
    // l_i / T + g_i and where it is (lowest index on ties); unused when decoding greedily
    float gs; int gidx;
    __device__ __forceinline__ void init() { m = -INFINITY; Z = 0.f; S = 0.f; idx = 0x7FFFFFFF; gs = -INFINITY; gidx = 0x7FFFFFFF; }
    __device__ __forceinline__ void merge(const EntStat &o) {
        if (o.Z == 0.f) return;                      // empty set
        if (Z == 0.f) { *this = o; return; }
        float M = fmaxf(m, o.m);
        float da = m - M, db = o.m - M;              // <= 0
        float ea = __expf(da), eb = __expf(db);
        float nS = ea * (S + da * Z) + eb * (o.S + db * o.Z);
        float nZ = ea * Z + eb * o.Z;
        if (o.m > m || (o.m == m && o.idx < idx)) idx = o.idx;
        if (o.gs > gs || (o.gs == gs && o.gidx < gidx)) { gs = o.gs; gidx = o.gidx; }
        m = M; Z = nZ; S = nS;
    }
};
__device__ __forceinline__ EntStat wave_merge(EntStat s) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        EntStat t;
        t.m = __shfl_xor(s.m, o, kWave); t.Z = __shfl_xor(s.Z, o, kWave);
        t.S = __shfl_xor(s.S, o, kWave); t.idx = __shfl_xor(s.idx, o, kWave);
        t.gs = __shfl_xor(s.gs, o, kWave); t.gidx = __shfl_xor(s.gidx, o, kWave);
        s.merge(t);
    }
    return s;
}

// ---- sampling noise ------------------------------------------------------------------
// Algorithm 1 samples y ~ softmax(l / T).  By the Gumbel-max identity that is
// argmax_i (l_i / T + g_i) with g_i = -ln(-ln u_i) and u_i independent uniforms on (0, 1),
// which folds into the LM head's running arg max: no pass over materialised logits.
// The uniforms are a pure function of (seed, sequence, token index, vocabulary index):
// Philox-4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3",
// SC 2011), key = seed, counter = (i / 4, token index, sequence, 0), word i % 4;
// u = (2k + 1) / 2^24 with k the word's top 23 bits (exact in fp32, never 0 or 1).
struct Philox4 { uint32_t x, y, z, w; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
    constexpr uint32_t kMul0 = 0xD2511F53u, kMul1 = 0xCD9E8D57u, kWeyl0 = 0x9E3779B9u, kWeyl1 = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(kMul0, c0), lo0 = kMul0 * c0;
        const uint32_t hi1 = __umulhi(kMul1, c2), lo1 = kMul1 * c2;
        c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
        k0 += kWeyl0; k1 += kWeyl1;
    }
    return Philox4{c0, c1, c2, c3};
}

__device__ __forceinline__ float gumbel_noise(uint32_t k0, uint32_t k1, int seq, int token_index, int i) {
    const Philox4 r = philox4x32_10((uint32_t)i >> 2, (uint32_t)token_index, (uint32_t)seq, 0u, k0, k1);
    const int lane = i & 3;
    const uint32_t word = lane == 0 ? r.x : (lane == 1 ? r.y : (lane == 2 ? r.z : r.w));
    const float u = (float)(2u * (word >> 9) + 1u) * (1.0f / 16777216.0f);
    return -logf(-logf(u));
}

}  // namespace ead
