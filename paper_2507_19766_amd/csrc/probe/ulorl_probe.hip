// ulorl_probe: a torch-free driver for profiling the token-loss kernels under rocprofv3.
//
// Allocates a synthetic [N, V] bf16 logits tensor with hipMalloc, fills it on the device with
// hashed pseudo-Gaussian values (a fraction of rows gets one boosted logit, and the chosen token
// of such a row is the boosted one), then runs, `iters` times:
//   1. plain_copy_kernel   reads N*V*2 bytes and writes N*V*2 bytes: the reference dispatch of
//                          KNOWN size that hardware byte counters are scaled by;
//   2. ulorl_token_loss_fwd   (row statistics + O(N) epilogue);
//   3. ulorl_token_loss_bwd   (in place unless --out-of-place);
//   4. plain_copy_kernel again (restores the logits), then ulorl_token_loss_fwd_bwd, the one-call
//      fused path (in place unless --out-of-place).
// It prints HIP-event timings per call.  It exists because counter collection needs a process
// that issues nothing but plain kernel dispatches.
//
// With --gemm M N K it instead times ulorl_gemm_tn_bf16 (the MFMA product of the lm_head variant)
// on hashed operands, for matrix-core counters.
//
// usage: ulorl_probe [--rows N] [--vocab V] [--iters K] [--out-of-place] [--spike F]
//        ulorl_probe --gemm M N K [--tile I] [--pad P] [--zeros] [--iters K]
//        (any form: --tune KNOB VALUE, repeated, sets launch-shape knobs first)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ulorl.h"

#define CHECK(x)                                                                            \
    do {                                                                                    \
        hipError_t e_ = (x);                                                                \
        if (e_ != hipSuccess) {                                                             \
            std::fprintf(stderr, "%s:%d %s\n", __FILE__, __LINE__, hipGetErrorString(e_));  \
            std::exit(1);                                                                   \
        }                                                                                   \
    } while (0)

namespace {

__device__ __forceinline__ uint32_t mix(uint64_t x)
{
    x ^= x >> 33; x *= 0xff51afd7ed558ccdULL;
    x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL;
    x ^= x >> 33;
    return (uint32_t)x;
}

// sum of four uniform bytes, centred and scaled: variance 1 to within a few per cent
__device__ __forceinline__ float rough_normal(uint32_t h)
{
    const float s = (float)(h & 255u) + (float)((h >> 8) & 255u) + (float)((h >> 16) & 255u) + (float)(h >> 24);
    return (s - 510.0f) * (1.0f / 147.8f);
}

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__global__ void fill_kernel(uint16_t* z, int32_t* y, float* adv, int64_t N, int32_t V, float std_, float boost,
                            uint32_t spike_permille)
{
    const int64_t row = blockIdx.x;
    const uint32_t hr = mix(0x9e3779b97f4a7c15ULL * (uint64_t)(row + 1));
    const bool spiked = (hr % 1000u) < spike_permille;
    const int32_t where = (int32_t)(mix(hr + 77u) % (uint32_t)V);
    for (int32_t j = threadIdx.x; j < V; j += blockDim.x) {
        float v = std_ * rough_normal(mix(((uint64_t)row << 32) | (uint32_t)j));
        if (spiked && j == where) v += boost;
        z[row * (int64_t)V + j] = to_bf16(v);
    }
    if (threadIdx.x == 0) {
        y[row] = spiked ? where : (int32_t)(mix(hr + 5u) % (uint32_t)V);
        adv[row] = 1.0f;
    }
}

__global__ void fill_bf16_kernel(uint16_t* p, int64_t n, uint64_t salt)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) p[i] = to_bf16(rough_normal(mix(salt + (uint64_t)i)));
}

__global__ void perturb_kernel(const float* logp, float* old_logp, int64_t N)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < N) old_logp[t] = logp[t] + 0.1f * rough_normal(mix(0x1234567ULL + (uint64_t)t));
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ void plain_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t nvec)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (; i < nvec; i += step) dst[i] = src[i];
}

float ms_between(hipEvent_t a, hipEvent_t b)
{
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, a, b));
    return ms;
}

}  // namespace

int main(int argc, char** argv)
{
    int64_t N = 16384;
    int64_t V = 151936;
    int iters = 3;
    bool inplace = true;
    int spike = 400;
    int64_t gm = 0, gn = 0, gk = 0;
    int tile = -1;
    int64_t pad = 0;     // --gemm only: extra elements in the operands' leading dimensions
    bool zeros = false;  // --gemm only: all-zero operands (the matrix pipes switch the least: the clock is at its highest)
    for (int i = 1; i < argc; ++i) {
        if (!std::strcmp(argv[i], "--gemm") && i + 3 < argc) {
            gm = std::atoll(argv[i + 1]); gn = std::atoll(argv[i + 2]); gk = std::atoll(argv[i + 3]);
            i += 3;
            continue;
        }
        if (!std::strcmp(argv[i], "--tile") && i + 1 < argc) { tile = std::atoi(argv[++i]); continue; }
        if (!std::strcmp(argv[i], "--pad") && i + 1 < argc) { pad = std::atoll(argv[++i]); continue; }
        if (!std::strcmp(argv[i], "--zeros")) { zeros = true; continue; }
        if (!std::strcmp(argv[i], "--tune") && i + 2 < argc) {     // --tune KNOB VALUE (ulorl_tune)
            if (ulorl_tune(std::atoi(argv[i + 1]), std::atoi(argv[i + 2])) != ULORL_OK) { std::fprintf(stderr, "bad --tune\n"); return 2; }
            i += 2;
            continue;
        }
        if (!std::strcmp(argv[i], "--rows") && i + 1 < argc) N = std::atoll(argv[++i]);
        else if (!std::strcmp(argv[i], "--vocab") && i + 1 < argc) V = std::atoll(argv[++i]);
        else if (!std::strcmp(argv[i], "--iters") && i + 1 < argc) iters = std::atoi(argv[++i]);
        else if (!std::strcmp(argv[i], "--spike") && i + 1 < argc) spike = std::atoi(argv[++i]);
        else if (!std::strcmp(argv[i], "--out-of-place")) inplace = false;
        else { std::fprintf(stderr, "unknown argument %s\n", argv[i]); return 2; }
    }
    if (N <= 0 || V <= 0 || V % 8 != 0 || iters <= 0) { std::fprintf(stderr, "need N>0, V>0 multiple of 8\n"); return 2; }
    if (gm > 0) {
        if (tile >= 0 && ulorl_tune(ULORL_TUNE_GEMM_TILE, tile) != ULORL_OK) { std::fprintf(stderr, "bad tile\n"); return 2; }
        uint16_t *a = nullptr, *b = nullptr;
        float* c = nullptr;
        if (pad < 0 || pad % 8 != 0) { std::fprintf(stderr, "--pad must be a non-negative multiple of 8\n"); return 2; }
        const int64_t ld = gk + pad;
        CHECK(hipMalloc(&a, (size_t)gm * ld * 2)); CHECK(hipMalloc(&b, (size_t)gn * ld * 2)); CHECK(hipMalloc(&c, (size_t)gm * gn * 4));
        if (zeros) {
            CHECK(hipMemset(a, 0, (size_t)gm * ld * 2));
            CHECK(hipMemset(b, 0, (size_t)gn * ld * 2));
        } else {
            hipLaunchKernelGGL(fill_bf16_kernel, dim3(4096), dim3(256), 0, 0, a, gm * ld, 11ULL << 40);
            hipLaunchKernelGGL(fill_bf16_kernel, dim3(4096), dim3(256), 0, 0, b, gn * ld, 12ULL << 40);
        }
        CHECK(hipDeviceSynchronize());
        hipEvent_t e0, e1;
        CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
        double tot = 0;
        for (int it = 0; it < iters + 1; ++it) {
            CHECK(hipEventRecord(e0, 0));
            const int rc = ulorl_gemm_tn_bf16(a, ld, b, ld, gm, gn, gk, c, gn, nullptr);
            if (rc != ULORL_OK) { std::fprintf(stderr, "gemm: %s\n", ulorl_status_string(rc)); return 1; }
            CHECK(hipEventRecord(e1, 0));
            CHECK(hipDeviceSynchronize());
            if (it > 0) tot += ms_between(e0, e1);
        }
        const double ms = tot / iters;
        std::printf("gemm_tn_bf16 %lld x %lld x %lld (ld %lld) tile %d: %.3f ms  %.1f TFLOP/s\n", (long long)gm,
                    (long long)gn, (long long)gk, (long long)ld, tile, ms, 2.0 * gm * gn * gk / ms / 1e9);
        return 0;
    }

    const size_t bytes = (size_t)N * (size_t)V * 2;
    uint16_t *z = nullptr, *pristine = nullptr, *dz = nullptr;
    CHECK(hipMalloc(&z, bytes));
    CHECK(hipMalloc(&pristine, bytes));
    if (!inplace) CHECK(hipMalloc(&dz, bytes));
    int32_t *y = nullptr, *cu = nullptr;
    float *adv, *old_logp, *loss, *logp, *ent, *lse, *g;
    int64_t* counters;
    void* ws;
    const size_t ws_bytes = ulorl_token_loss_workspace_bytes(N, V, 1);
    CHECK(hipMalloc(&y, N * 4)); CHECK(hipMalloc(&cu, 8));
    CHECK(hipMalloc(&adv, N * 4)); CHECK(hipMalloc(&old_logp, N * 4)); CHECK(hipMalloc(&loss, 4));
    CHECK(hipMalloc(&logp, N * 4)); CHECK(hipMalloc(&ent, N * 4)); CHECK(hipMalloc(&lse, N * 4));
    CHECK(hipMalloc(&g, N * 4)); CHECK(hipMalloc(&counters, 32)); CHECK(hipMalloc(&ws, ws_bytes));
    const int32_t cu_host[2] = {0, (int32_t)N};
    CHECK(hipMemcpy(cu, cu_host, 8, hipMemcpyHostToDevice));

    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)N), dim3(256), 0, 0, pristine, y, adv, N, (int32_t)V, 3.0f, 15.0f,
                       (uint32_t)spike);
    CHECK(hipGetLastError());
    const int64_t nvec = (int64_t)(bytes / 16);
    hipLaunchKernelGGL(plain_copy_kernel, dim3(256 * 32), dim3(256), 0, 0, (const u32x4*)pristine, (u32x4*)z, nvec);

    ulorl_params p = {};
    p.eps_low = p.eps_high = 0.2f; p.tau = 0.99f; p.sigma = 0.2f;
    p.is_mode = ULORL_IS_SAIS; p.gate_mode = ULORL_GATE_ALWAYS; p.seg_len = 16384;
    // record old log-probs with a stats-only pass, then perturb them
    int rc = ulorl_token_loss_fwd(z, ULORL_BF16, N, V, V, y, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr,
                                  logp, ent, lse, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr);
    if (rc != ULORL_OK) { std::fprintf(stderr, "stats pass: %s\n", ulorl_status_string(rc)); return 1; }
    hipLaunchKernelGGL(perturb_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, 0, logp, old_logp, N);
    CHECK(hipDeviceSynchronize());

    hipEvent_t ev[6];
    for (auto& e : ev) CHECK(hipEventCreate(&e));
    double t_copy = 0, t_fwd = 0, t_bwd = 0, t_fused = 0;
    for (int it = 0; it < iters; ++it) {
        CHECK(hipEventRecord(ev[0], 0));
        hipLaunchKernelGGL(plain_copy_kernel, dim3(256 * 32), dim3(256), 0, 0, (const u32x4*)pristine, (u32x4*)z, nvec);
        CHECK(hipEventRecord(ev[1], 0));
        rc = ulorl_token_loss_fwd(z, ULORL_BF16, N, V, V, y, cu, 1, nullptr, old_logp, adv, &p, loss, logp, ent, lse, g,
                                  nullptr, nullptr, nullptr, nullptr, nullptr, counters, ws, ws_bytes, nullptr);
        if (rc != ULORL_OK) { std::fprintf(stderr, "fwd: %s\n", ulorl_status_string(rc)); return 1; }
        CHECK(hipEventRecord(ev[2], 0));
        rc = ulorl_token_loss_bwd(z, ULORL_BF16, N, V, V, y, lse, g, 1.0f, inplace ? (void*)z : (void*)dz, nullptr);
        if (rc != ULORL_OK) { std::fprintf(stderr, "bwd: %s\n", ulorl_status_string(rc)); return 1; }
        CHECK(hipEventRecord(ev[3], 0));
        hipLaunchKernelGGL(plain_copy_kernel, dim3(256 * 32), dim3(256), 0, 0, (const u32x4*)pristine, (u32x4*)z, nvec);
        CHECK(hipEventRecord(ev[4], 0));
        rc = ulorl_token_loss_fwd_bwd(z, ULORL_BF16, N, V, V, y, cu, 1, nullptr, old_logp, adv, &p, 1.0f, loss, logp, ent,
                                      lse, g, nullptr, nullptr, nullptr, nullptr, nullptr, counters,
                                      inplace ? (void*)z : (void*)dz, ws, ws_bytes, nullptr);
        if (rc != ULORL_OK) { std::fprintf(stderr, "fwd_bwd: %s\n", ulorl_status_string(rc)); return 1; }
        CHECK(hipEventRecord(ev[5], 0));
        CHECK(hipDeviceSynchronize());
        t_copy += ms_between(ev[0], ev[1]);
        t_fwd += ms_between(ev[1], ev[2]);
        t_bwd += ms_between(ev[2], ev[3]);
        t_fused += ms_between(ev[4], ev[5]);
    }
    std::vector<float> gh(N);
    int64_t cnt[4];
    float lossh;
    CHECK(hipMemcpy(gh.data(), g, N * 4, hipMemcpyDeviceToHost));
    CHECK(hipMemcpy(cnt, counters, 32, hipMemcpyDeviceToHost));
    CHECK(hipMemcpy(&lossh, loss, 4, hipMemcpyDeviceToHost));
    int64_t live = 0;
    for (float v : gh) live += v != 0.0f;
    const double gb = bytes / 1e9;
    std::printf("rows %lld vocab %lld bf16 (%.3f GB per pass), %s, %d iterations\n", (long long)N, (long long)V, gb,
                inplace ? "in place" : "out of place", iters);
    std::printf("loss %.6f masked %lld clipped %lld live_rows %lld status %lld\n", lossh, (long long)cnt[0],
                (long long)cnt[1], (long long)live, (long long)cnt[3]);
    std::printf("plain_copy_kernel : %8.3f ms  %7.1f GB/s  (read %.3f GB + write %.3f GB)\n", t_copy / iters,
                2 * gb / (t_copy / iters) * 1e3, gb, gb);
    std::printf("token_loss_fwd    : %8.3f ms  %7.1f GB/s  (read %.3f GB)\n", t_fwd / iters, gb / (t_fwd / iters) * 1e3, gb);
    const double bwd_gb = gb * (double)(N + live) / (double)N;
    std::printf("token_loss_bwd    : %8.3f ms  %7.1f GB/s  (%.3f GB algorithmic)\n", t_bwd / iters,
                bwd_gb / (t_bwd / iters) * 1e3, bwd_gb);
    std::printf("token_loss_fwd_bwd: %8.3f ms  %7.1f GB/s  (read %.3f GB + write %.3f GB)\n", t_fused / iters,
                2 * gb / (t_fused / iters) * 1e3, gb, gb);
    return 0;
}
