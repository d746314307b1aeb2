// Torch-free driver for hardware-counter runs (built by `python bench.py --build-probe`): builds the
// Llama-1B / Llama-8B or the Qwen-0.5B / Qwen-14B shaped pair with constant weights straight through
// the C ABI, decodes a few steps with each model, and runs one plain copy kernel of known size as the
// reference point for byte counters.  Values do not matter for traffic, only shapes do.
//   rocprofv3 --pmc FETCH_SIZE --output-format csv -d out -- ./roofline_probe [pair] [steps] [batch] [prompt_len]
// pair: llama (default) or qwen.  batch > 1 decodes that many identical rows together (the
// matrix-core path of the linear layers), for counters of the batched kernels.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include <string.h>

#include "include/ead.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } } while (0)

__global__ void k_fill_u16(uint16_t *p, size_t n, uint16_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void k_fill_f32(float *p, size_t n, float v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
// plain copy of n 16-byte words: reads 16n bytes, writes 16n bytes
__global__ void k_copy_probe(const uint4 *src, uint4 *dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

struct Shape { int L, d, H, KV, F, V; float eps, theta; };

static void *dev_bf16(size_t n, uint16_t v) {
    void *p; CK(hipMalloc(&p, n * 2));
    hipLaunchKernelGGL(k_fill_u16, dim3(4096), dim3(256), 0, 0, (uint16_t *)p, n, v);
    return p;
}
static float *dev_f32(size_t n, float v) {
    float *p; CK(hipMalloc(&p, n * 4));
    hipLaunchKernelGGL(k_fill_f32, dim3(256), dim3(256), 0, 0, p, n, v);
    return p;
}

struct Built { ead_model_desc d; std::vector<const void *> wq, wk, wv, wo, wg, wu, wd; std::vector<const float *> na, nf; };

static void build(const Shape &s, Built &b) {
    const int hd = s.d / s.H;
    const uint16_t w = 0x3c23;   // bf16 0.00995
    b.d = ead_model_desc{};
    b.d.n_layers = s.L; b.d.d_model = s.d; b.d.n_heads = s.H; b.d.n_kv_heads = s.KV; b.d.head_dim = hd; b.d.d_ffn = s.F;
    b.d.vocab = s.V; b.d.rms_eps = s.eps; b.d.rope_theta = s.theta; b.d.dtype = EAD_BF16;
    b.d.embed = dev_bf16((size_t)s.V * s.d, w);
    b.d.lm_head = dev_bf16((size_t)s.V * s.d, w);
    b.d.norm_final = dev_f32(s.d, 1.f);
    for (int l = 0; l < s.L; ++l) {
        b.wq.push_back(dev_bf16((size_t)s.H * hd * s.d, w)); b.wk.push_back(dev_bf16((size_t)s.KV * hd * s.d, w));
        b.wv.push_back(dev_bf16((size_t)s.KV * hd * s.d, w)); b.wo.push_back(dev_bf16((size_t)s.d * s.H * hd, w));
        b.wg.push_back(dev_bf16((size_t)s.F * s.d, w)); b.wu.push_back(dev_bf16((size_t)s.F * s.d, w));
        b.wd.push_back(dev_bf16((size_t)s.d * s.F, w));
        b.na.push_back(dev_f32(s.d, 1.f)); b.nf.push_back(dev_f32(s.d, 1.f));
    }
    b.d.wq = b.wq.data(); b.d.wk = b.wk.data(); b.d.wv = b.wv.data(); b.d.wo = b.wo.data();
    b.d.w_gate = b.wg.data(); b.d.w_up = b.wu.data(); b.d.w_down = b.wd.data();
    b.d.norm_attn = b.na.data(); b.d.norm_ffn = b.nf.data();
}

int main(int argc, char **argv) {
    const char *pair = argc > 1 ? argv[1] : "llama";
    const int steps = argc > 2 ? atoi(argv[2]) : 4;
    const int batch = argc > 3 ? atoi(argv[3]) : 1;
    const int prompt_len = argc > 4 ? atoi(argv[4]) : 512;
    const bool qwen = strcmp(pair, "qwen") == 0;
    if ((!qwen && strcmp(pair, "llama") != 0) || steps < 1 || batch < 1 || batch > 256 || prompt_len < 1 || prompt_len > 4096) {
        fprintf(stderr, "usage: roofline_probe [llama|qwen] [steps] [batch<=256] [prompt_len<=4096]\n"); return 2;
    }
    Built S, L;
    const int vocab = qwen ? 151936 : 128256;
    if (qwen) {
        build(Shape{24, 896, 14, 2, 4864, vocab, 1e-6f, 1e6f}, S);
        build(Shape{48, 5120, 40, 8, 13824, vocab, 1e-6f, 1e6f}, L);
    } else {
        build(Shape{16, 2048, 32, 8, 8192, vocab, 1e-5f, 5e5f}, S);
        build(Shape{32, 4096, 32, 8, 14336, vocab, 1e-5f, 5e5f}, L);
    }
    CK(hipDeviceSynchronize());
    ead_params p{5, 1e30f, 10, EAD_NATS, batch, prompt_len + 2 * steps + 8, -1, nullptr};
    ead_handle *h = nullptr;
    if (ead_create(&S.d, &L.d, &p, &h) != EAD_OK) { fprintf(stderr, "ead_create: %s\n", ead_last_error(nullptr)); return 1; }
    // reference copy: 1 GiB read + 1 GiB written
    {
        const size_t n = (size_t)1 << 26;
        uint4 *a, *b; CK(hipMalloc(&a, n * 16)); CK(hipMalloc(&b, n * 16));
        CK(hipMemset(a, 1, n * 16));
        hipLaunchKernelGGL(k_copy_probe, dim3(2048), dim3(256), 0, 0, a, b, n);
        CK(hipDeviceSynchronize());
        CK(hipFree(a)); CK(hipFree(b));
    }
    std::vector<int32_t> prompt((size_t)prompt_len * batch);
    for (size_t i = 0; i < prompt.size(); ++i) prompt[i] = (int32_t)((i * 7919) % vocab);
    std::vector<int32_t> lens(batch, prompt_len);
    for (int which = 0; which < 2; ++which) {
        if (ead_force_model(h, which) != EAD_OK || ead_begin(h, prompt.data(), lens.data(), batch, steps) != EAD_OK ||
            ead_decode(h, steps) != EAD_OK) { fprintf(stderr, "decode: %s\n", ead_last_error(h)); return 1; }
    }
    ead_stats st; ead_get_stats(h, &st);
    printf("probe done: %d steps per model, batch %d, last run large tokens %lld\n", steps, batch, (long long)st.tokens_large);
    ead_destroy(h);
    return 0;
}
