// The small neighbours of the token loss: the pool update of the segment-rollout loop and the
// advantage preparation (the steps just before it) and per-segment training-dynamics diagnostics
// (read off its outputs).  All are bandwidth-trivial; they exist so that a training step needs no
// host round trip between rollout bookkeeping, reward and gradient.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ulorl.h"
#include "ulorl_internal.hpp"

using namespace ulorl_detail;

#pragma clang fp contract(off)

namespace {

constexpr int kBlock = 1024;

__device__ __forceinline__ double shfl_xor_f64(double x, int off)
{
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return __hiloint2double(hi, lo);
}

// Fixed-shape reductions over the workgroup: lanes by xor-shuffle, waves through LDS in order.
__device__ __forceinline__ double block_sum_f64(double x, double* scratch)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += shfl_xor_f64(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = x;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < kBlock / 64; ++w) s += scratch[w];
    return s;
}

// ---------------------------------------------------------------------------------------------
// advantage preparation (Eq. 4; dynamic-sampling constraint of Eq. 7; Sec. 3.5)
// ---------------------------------------------------------------------------------------------
// One workgroup walks all groups (a step has ~10^2..10^3 of them).
__global__ __launch_bounds__(kBlock) void group_advantage_kernel(const float* __restrict__ rewards,
                                                                 const uint8_t* __restrict__ truncated,
                                                                 const int32_t* __restrict__ cu, int32_t R, int32_t G,
                                                                 double eps, int unbiased, float* __restrict__ resp_adv,
                                                                 uint8_t* __restrict__ group_keep,
                                                                 int64_t* __restrict__ kept_tokens)
{
    __shared__ double scratch[kBlock / 64];
    const int ngroups = R / G;
    double kept = 0.0;   // exact in fp64 for any token count below 2^53
    for (int g = threadIdx.x; g < ngroups; g += kBlock) {
        const int g0 = g * G;
        double sum = 0.0;
        int correct = 0;
        for (int i = g0; i < g0 + G; ++i) {
            const double r = (truncated && truncated[i]) ? 0.0 : (double)rewards[i];
            sum += r;
            correct += r > 0.0;
        }
        const double mean = sum / G;
        double ss = 0.0;
        for (int i = g0; i < g0 + G; ++i) {
            const double r = (truncated && truncated[i]) ? 0.0 : (double)rewards[i];
            ss += (r - mean) * (r - mean);
        }
        const double denom = unbiased ? (G > 1 ? G - 1 : 1) : G;
        const double sd = sqrt(ss / denom);
        const bool keep = correct > 0 && correct < G;
        if (group_keep) group_keep[g] = keep ? 1 : 0;
        for (int i = g0; i < g0 + G; ++i) {
            const double r = (truncated && truncated[i]) ? 0.0 : (double)rewards[i];
            resp_adv[i] = keep ? (float)((r - mean) / (sd + eps)) : 0.0f;
            if (keep) kept += (double)((int64_t)cu[i + 1] - (int64_t)cu[i]);
        }
    }
    kept = block_sum_f64(kept, scratch);
    if (threadIdx.x == 0 && kept_tokens) *kept_tokens = (int64_t)kept;
}

__global__ __launch_bounds__(256) void broadcast_advantage_kernel(const float* __restrict__ resp_adv,
                                                                  const int32_t* __restrict__ cu, int32_t R, int64_t N,
                                                                  float* __restrict__ token_adv)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= N) return;
    int lo = 0, hi = R;   // largest i with cu[i] <= t
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)cu[mid] <= t) lo = mid; else hi = mid;
    }
    token_adv[t] = resp_adv[lo];
}

// ---------------------------------------------------------------------------------------------
// per-segment diagnostics (standalone form; the forward calls produce the same numbers as a
// by-product through the same device functions, segment_stats.hpp)
// ---------------------------------------------------------------------------------------------
struct DiagInputs {
    const int32_t* seg;
    const float* ratio;
    const float* logp;
    const float* old_logp;
    const float* entropy;
    const uint8_t* mask;
    const float* adv;
    int64_t N;
    double eps_low, eps_high;
};

__global__ __launch_bounds__(kSegBlock) void segment_partial_kernel(DiagInputs in, SegStatsArgs a)
{
    extern __shared__ double seg_table[];
    const int64_t t = (int64_t)blockIdx.x * kSegBlock + threadIdx.x;
    const bool valid = t < in.N;
    int k;
    double v[kSegStats], oor;
    seg_token_values(valid, valid ? in.seg[t] : 0, a.K, valid ? in.ratio[t] : 0.0f, valid ? in.logp[t] : 0.0f,
                     in.old_logp != nullptr, (valid && in.old_logp) ? in.old_logp[t] : 0.0f, valid ? in.entropy[t] : 0.0f,
                     valid ? in.mask[t] : (uint8_t)0, valid ? in.adv[t] : 0.0f, in.eps_low, in.eps_high, k, v, oor);
    const double o = seg_block_partials(k, v, oor, a.K, seg_table, a.part + (int64_t)blockIdx.x * a.K * kSegStats);
    if (threadIdx.x == 0) a.part_oor[blockIdx.x] = o;
}

__global__ __launch_bounds__(kSegBlock) void segment_final_kernel(SegStatsArgs a, int64_t nblk)
{
    __shared__ double scratch[kSegBlock];
    seg_finalize(a, nblk, scratch);
}

// ---------------------------------------------------------------------------------------------
// segment-rollout pool update (Algorithm 1, Sec. 3.1.1)
// ---------------------------------------------------------------------------------------------
// Inclusive prefix sum over the workgroup (wave scans by shuffle, wave totals through LDS in
// index order).  Returns the thread's inclusive sum; *total = sum over the workgroup.
__device__ __forceinline__ int block_scan_i32(int v, int* wave_tot, int* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(v, off);
        if (lane >= off) v += up;
    }
    __syncthreads();                 // wave_tot may still be read from the previous scan
    if (lane == 63) wave_tot[wave] = v;
    __syncthreads();
    int before = 0, all = 0;
    for (int w = 0; w < kBlock / 64; ++w) {
        const int x = wave_tot[w];
        before += w < wave ? x : 0;
        all += x;
    }
    *total = all;
    return v + before;
}

// One workgroup walks the samples in blocks of 1024: classify (the three ways a decode ends),
// then place each sample by an order-preserving prefix sum.
__global__ __launch_bounds__(kBlock) void pool_step_kernel(int32_t B, const int32_t* __restrict__ prev_len,
                                                           const int32_t* __restrict__ new_len,
                                                           const uint8_t* __restrict__ hit_eos, int32_t seg_len,
                                                           int32_t max_len, uint8_t* __restrict__ state,
                                                           int32_t* __restrict__ total_len,
                                                           int32_t* __restrict__ segments,
                                                           int32_t* __restrict__ unfinished_idx,
                                                           int32_t* __restrict__ experience_idx,
                                                           int32_t* __restrict__ exp_cu,
                                                           uint8_t* __restrict__ exp_truncated,
                                                           int64_t* __restrict__ counts)
{
    __shared__ int wave_tot[kBlock / 64];
    const int tid = threadIdx.x;
    int base_unf = 0, base_exp = 0, base_tok = 0, n_trunc = 0, n_bad = 0;
    if (tid == 0) exp_cu[0] = 0;
    for (int32_t c0 = 0; c0 < B; c0 += kBlock) {
        const int32_t i = c0 + tid;
        int st = 0, bad = 0, t = 0, f_unf = 0, f_exp = 0;
        if (i < B) {
            int64_t p = prev_len[i], n = new_len[i];
            if (p < 0 || p >= max_len) { bad = 1; p = p < 0 ? 0 : max_len - 1; }
            int64_t room = (int64_t)max_len - p;
            if (room > seg_len) room = seg_len;
            if (n < 0 || n > room) { bad = 1; n = n < 0 ? 0 : room; }
            t = (int)(p + n);
            const bool eos_flag = hit_eos[i] != 0;
            if (eos_flag && n == 0) bad = 1;
            if (bad) st = 0;
            else if (eos_flag) st = 1;
            else if (t >= max_len) st = 2;
            else if (n == seg_len) st = 0;
            else { st = 0; bad = 1; }
            state[i] = (uint8_t)st;
            total_len[i] = t;
            segments[i] = t == 0 ? 0 : (t + seg_len - 1) / seg_len;
            f_unf = st == 0;
            f_exp = st != 0;
        }
        int tot_unf, tot_exp, tot_tok, tot_trunc, tot_bad;
        const int in_unf = block_scan_i32(f_unf, wave_tot, &tot_unf);
        const int in_exp = block_scan_i32(f_exp, wave_tot, &tot_exp);
        const int in_tok = block_scan_i32(f_exp ? t : 0, wave_tot, &tot_tok);
        block_scan_i32(st == 2, wave_tot, &tot_trunc);
        block_scan_i32(bad, wave_tot, &tot_bad);
        if (f_unf) unfinished_idx[base_unf + in_unf - 1] = i;
        if (f_exp) {
            const int slot = base_exp + in_exp - 1;
            experience_idx[slot] = i;
            exp_truncated[slot] = (uint8_t)(st == 2);
            exp_cu[slot + 1] = base_tok + in_tok;
        }
        base_unf += tot_unf; base_exp += tot_exp; base_tok += tot_tok; n_trunc += tot_trunc; n_bad += tot_bad;
    }
    if (tid == 0) {
        counts[0] = base_unf; counts[1] = base_exp; counts[2] = n_trunc; counts[3] = base_tok; counts[4] = n_bad;
    }
}

}  // namespace

extern "C" {

int32_t ulorl_advantage_prep(const float* rewards, const uint8_t* truncated, const int32_t* cu_seqlens, int32_t R,
                             int32_t group_size, int64_t N, float eps, int32_t unbiased, float* resp_adv,
                             uint8_t* group_keep, float* token_adv, int64_t* kept_tokens, void* hip_stream)
{
    if (!rewards || !cu_seqlens || !resp_adv || !token_adv) return ULORL_ERR_NULL;
    if (R <= 0 || group_size <= 0 || R % group_size != 0 || N <= 0 || N > 0x7fffffffLL) return ULORL_ERR_SHAPE;
    if (!(eps >= 0.0f)) return ULORL_ERR_PARAM;
    hipStream_t st = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(group_advantage_kernel, dim3(1), dim3(kBlock), 0, st, rewards, truncated, cu_seqlens, R, group_size,
                       (double)eps, unbiased ? 1 : 0, resp_adv, group_keep, kept_tokens);
    hipLaunchKernelGGL(broadcast_advantage_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, resp_adv, cu_seqlens,
                       R, N, token_adv);
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

size_t ulorl_segment_diagnostics_workspace_bytes(int64_t N, int32_t K)
{
    if (N <= 0 || N > 0x7fffffffLL || K <= 0 || K > kSegMaxK) return 0;
    return seg_workspace_bytes(N, K);
}

int32_t ulorl_segment_diagnostics(int64_t N, int32_t K, const int32_t* segment_ids, const float* ratio,
                                  const float* logp, const float* old_logp, const float* entropy,
                                  const uint8_t* mpt_mask, const float* advantages, float eps_low, float eps_high,
                                  int64_t* count, double* ratio_sum, float* ratio_max, int64_t* clipped,
                                  double* kl_sum, double* ent_sum, int64_t* masked, int64_t* out_of_range,
                                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!segment_ids || !ratio || !logp || !entropy || !mpt_mask || !advantages) return ULORL_ERR_NULL;
    if (N <= 0) return ULORL_ERR_SHAPE;
    if (!(eps_low >= 0.0f) || !(eps_high >= 0.0f)) return ULORL_ERR_PARAM;
    ulorl_segment_stats st = {};
    st.K = K;
    st.count = count; st.ratio_sum = ratio_sum; st.ratio_max = ratio_max; st.clipped = clipped;
    st.kl_sum = kl_sum; st.ent_sum = ent_sum; st.masked = masked; st.out_of_range = out_of_range;
    st.workspace = workspace; st.workspace_bytes = workspace_bytes;
    SegStatsArgs a;
    const int32_t rc = resolve_segment_stats(&st, N, &a);
    if (rc != ULORL_OK) return rc;
    const int64_t nblk = (N + kSegBlock - 1) / kSegBlock;
    DiagInputs in;
    in.seg = segment_ids; in.ratio = ratio; in.logp = logp; in.old_logp = old_logp; in.entropy = entropy;
    in.mask = mpt_mask; in.adv = advantages; in.N = N;
    in.eps_low = (double)eps_low; in.eps_high = (double)eps_high;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(segment_partial_kernel, dim3((unsigned)nblk), dim3(kSegBlock), (size_t)K * kSegStats * sizeof(double),
                       stream, in, a);
    hipLaunchKernelGGL(segment_final_kernel, dim3(1), dim3(kSegBlock), 0, stream, a, nblk);
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

int32_t ulorl_segment_pool_step(int32_t B, const int32_t* prev_len, const int32_t* new_len, const uint8_t* hit_eos,
                                int32_t seg_len, int32_t max_len, uint8_t* state, int32_t* total_len,
                                int32_t* segments, int32_t* unfinished_idx, int32_t* experience_idx,
                                int32_t* exp_cu_seqlens, uint8_t* exp_truncated, int64_t* counts, void* hip_stream)
{
    if (!prev_len || !new_len || !hit_eos || !state || !total_len || !segments || !unfinished_idx || !experience_idx ||
        !exp_cu_seqlens || !exp_truncated || !counts)
        return ULORL_ERR_NULL;
    if (B <= 0 || seg_len <= 0 || max_len <= 0) return ULORL_ERR_SHAPE;
    if ((int64_t)B * (int64_t)max_len > 0x7fffffffLL) return ULORL_ERR_SHAPE;   // packed-batch offsets are int32
    hipLaunchKernelGGL(pool_step_kernel, dim3(1), dim3(kBlock), 0, (hipStream_t)hip_stream, B, prev_len, new_len, hit_eos,
                       seg_len, max_len, state, total_len, segments, unfinished_idx, experience_idx, exp_cu_seqlens,
                       exp_truncated, counts);
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

}  // extern "C"
