// Small stand-alone consumer of the C ABI for hardware-counter runs (no Python, no PyTorch): an 8B-shaped
// decoder with few layers and synthetic weights, a short prefill through the matrix-core append path, a few
// single-row decoding steps and one interrupt, then three plain device-to-device copy kernels of known size
// that calibrate the byte counters.  The values of the weights do not matter for traffic; they are small and
// finite.  Usage: traffic_probe [layers] [prompt tokens] [decode steps]
#include "include/asynclm.h"

#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

// bf16 values in about [-0.03, 0.03] from a counter hash
__global__ void k_fill_bf16(uint16_t* p, size_t n, uint32_t salt) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t h = (uint32_t)i * 2654435761u + salt;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        const float v = ((float)(h & 0xffff) - 32768.f) * (0.03f / 32768.f);
        p[i] = (uint16_t)(__float_as_uint(v) >> 16);
    }
}

__global__ void k_fill_f32(float* p, size_t n, float v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// the calibration kernel: reads n 16-byte words and writes them once
__global__ void k_plain_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

int main(int argc, char** argv) {
    const int layers = argc > 1 ? std::atoi(argv[1]) : 2;
    const int prompt = argc > 2 ? std::atoi(argv[2]) : 1024;
    const int steps = argc > 3 ? std::atoi(argv[3]) : 8;
    asynclm_config cfg{};
    cfg.n_layers = layers; cfg.d_model = 4096; cfg.n_q_heads = 32; cfg.n_kv_heads = 8; cfg.head_dim = 128;
    cfg.ffn = 14336; cfg.vocab = 128256; cfg.rms_eps = 1e-5f; cfg.rope_theta = 500000.f;
    cfg.dtype = ASYNCLM_DTYPE_BF16; cfg.max_seqs = 1; cfg.max_positions = prompt + steps + 64; cfg.kv_format = ASYNCLM_KV_AUTO;

    auto bf16 = [&](size_t n, uint32_t salt, void** out) -> int {
        CK(hipMalloc(out, n * 2));
        hipLaunchKernelGGL(k_fill_bf16, dim3(2048), dim3(256), 0, 0, (uint16_t*)*out, n, salt);
        return 0;
    };
    auto ones = [&](size_t n, void** out) -> int {
        CK(hipMalloc(out, n * 4));
        hipLaunchKernelGGL(k_fill_f32, dim3(64), dim3(256), 0, 0, (float*)*out, n, 1.f);
        return 0;
    };
    const size_t d = cfg.d_model, F = cfg.ffn, V = cfg.vocab, nq = (size_t)(cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim;
    void *embed, *head, *fnorm;
    if (bf16(V * d, 1, &embed) || bf16(V * d, 2, &head) || ones(d, &fnorm)) return 1;
    std::vector<const float*> an(layers), fn(layers);
    std::vector<const void*> wqkv(layers), wo(layers), wgu(layers), wd(layers);
    for (int l = 0; l < layers; ++l) {
        void* p;
        if (ones(d, &p)) return 1; an[l] = (const float*)p;
        if (ones(d, &p)) return 1; fn[l] = (const float*)p;
        if (bf16(nq * d, 10 + 4 * l, &p)) return 1; wqkv[l] = p;
        if (bf16(d * d, 11 + 4 * l, &p)) return 1; wo[l] = p;
        if (bf16(2 * F * d, 12 + 4 * l, &p)) return 1; wgu[l] = p;
        if (bf16(d * F, 13 + 4 * l, &p)) return 1; wd[l] = p;
    }
    CK(hipDeviceSynchronize());
    asynclm_weights w{};
    w.embed = embed; w.final_norm = (const float*)fnorm; w.lm_head = head;
    w.attn_norm = an.data(); w.wqkv = wqkv.data(); w.wo = wo.data(); w.ffn_norm = fn.data(); w.wgate_up = wgu.data(); w.wdown = wd.data();

    hipStream_t stream;
    CK(hipStreamCreate(&stream));
    asynclm_ctx* ctx = nullptr;
    int rc = asynclm_create(&ctx, &cfg, &w, stream);
    if (rc) { std::fprintf(stderr, "asynclm_create: %s\n", asynclm_strerror(rc)); return 1; }
    asynclm_set_option(ctx, "graph", 0);        // plain launches: one counter record per kernel
    std::vector<int32_t> toks(prompt);
    for (int i = 0; i < prompt; ++i) toks[i] = (int32_t)((1103515245u * (unsigned)i + 12345u) % (unsigned)V);
    if ((rc = asynclm_prefill(ctx, 0, toks.data(), prompt))) { std::fprintf(stderr, "prefill: %s\n", asynclm_strerror(rc)); return 1; }
    int32_t tok = -1;
    for (int i = 0; i < steps; ++i)
        if ((rc = asynclm_decode_step(ctx, 0, -1, &tok))) { std::fprintf(stderr, "decode: %s\n", asynclm_strerror(rc)); return 1; }
    if ((rc = asynclm_inject_interrupt(ctx, 0, toks.data(), 24))) { std::fprintf(stderr, "inject: %s\n", asynclm_strerror(rc)); return 1; }
    asynclm_synchronize(ctx);

    const size_t copy_bytes = (size_t)1 << 30, n16 = copy_bytes / 16;
    void *src, *dst;
    CK(hipMalloc(&src, copy_bytes)); CK(hipMalloc(&dst, copy_bytes));
    hipLaunchKernelGGL(k_fill_f32, dim3(2048), dim3(256), 0, stream, (float*)src, copy_bytes / 4, 1.f);
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(k_plain_copy, dim3(4096), dim3(256), 0, stream, (const uint4*)src, (uint4*)dst, n16);
    CK(hipStreamSynchronize(stream));
    std::printf("traffic_probe: layers %d prompt %d steps %d last token %d; k_plain_copy reads and writes %zu bytes per launch\n",
                layers, prompt, steps, tok, copy_bytes);
    asynclm_destroy(ctx);
    return 0;
}
