// Per-segment training-dynamics diagnostics (Sec. 3.1.2: drift of the importance ratio of older
// segments, share of clipped tokens; Sec. 3.2: entropy and MPT share): device code shared by the
// O(N) epilogue of the forward calls, which produces them from the values it holds in registers,
// and by the standalone ulorl_segment_diagnostics call, which reads them back from a forward call's
// outputs.  Both go through the same functions in the same order, so they give the same bits.
//
// Per workgroup of kSegBlock consecutive tokens: a table [K][7] in LDS; the waves take turns in
// index order, each wave walks the distinct segment ids of its lanes (in order of the first lane
// holding one) and adds the wave's fixed-tree sums to the table.  No floating-point atomics: the
// result depends on the inputs only.
#ifndef ULORL_SEGMENT_STATS_HPP
#define ULORL_SEGMENT_STATS_HPP

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ulorl_detail {

constexpr int kSegBlock = 1024;     // tokens per workgroup (that of the O(N) epilogue)
constexpr int kSegStats = 7;        // count, ratio_sum, ratio_max, clipped, kl_sum, ent_sum, masked
constexpr int kSegMaxK = 1024;      // the table [K][7] of doubles has to fit the default LDS limit

struct SegStatsArgs {
    int32_t K;              // 0: diagnostics not wanted
    double* part;           // [nblk][K][7] workspace
    double* part_oor;       // [nblk] workspace
    int64_t* count;
    double* ratio_sum;
    float* ratio_max;
    int64_t* clipped;
    double* kl_sum;
    double* ent_sum;
    int64_t* masked;
    int64_t* out_of_range;  // may be NULL
};

__device__ __forceinline__ double seg_shfl_xor(double x, int off)
{
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return __hiloint2double(hi, lo);
}

// One token's seven values from what a forward call stores (fp32 ratio / log-probs / entropy,
// the mask byte, the advantage): v[] and its segment id k (-1: no token, or id outside [0, K),
// then *oor = 1).
__device__ __forceinline__ void seg_token_values(bool valid, int32_t seg, int32_t K, float ratio, float logp,
                                                 bool have_old, float old_logp, float entropy, uint8_t mask,
                                                 float adv, double eps_low, double eps_high, int& k, double (&v)[kSegStats],
                                                 double& oor)
{
    k = -1;
    oor = 0.0;
#pragma unroll
    for (int s = 0; s < kSegStats; ++s) v[s] = 0.0;
    if (!valid) return;
    if (seg < 0 || seg >= K) {
        oor = 1.0;
        return;
    }
    k = seg;
    const double r = (double)ratio;
    const double A = (double)adv;
    const double c = fmin(fmax(r, 1.0 - eps_low), 1.0 + eps_high);
    v[0] = 1.0;
    v[1] = r;
    v[2] = r;
    v[3] = (r * A <= c * A) ? 0.0 : 1.0;
    v[4] = have_old ? (double)old_logp - (double)logp : 0.0;
    v[5] = (double)entropy;
    v[6] = mask ? 1.0 : 0.0;
}

// Adds the workgroup's tokens to table (LDS, [K][7]) and writes it to out (global, [K][7]); returns
// the workgroup's count of out-of-range tokens on every thread.  All kSegBlock threads must call.
__device__ __forceinline__ double seg_block_partials(int k, const double (&v)[kSegStats], double oor, int32_t K,
                                                     double* table, double* __restrict__ out)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < K * kSegStats; i += kSegBlock) table[i] = 0.0;
    __syncthreads();
    for (int w = 0; w < kSegBlock / 64; ++w) {
        if (wave == w) {
            unsigned long long remaining = __ballot(k >= 0);
            while (remaining != 0ull) {
                const int leader = __ffsll((long long)remaining) - 1;
                const int key = __shfl(k, leader);
                const bool mine = k == key;
                double x[kSegStats];
#pragma unroll
                for (int s = 0; s < kSegStats; ++s) x[s] = mine ? v[s] : 0.0;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
                    for (int s = 0; s < kSegStats; ++s) {
                        const double other = seg_shfl_xor(x[s], off);
                        x[s] = (s == 2) ? fmax(x[s], other) : x[s] + other;
                    }
                }
                if (lane == leader) {
                    double* t = table + key * kSegStats;
#pragma unroll
                    for (int s = 0; s < kSegStats; ++s) t[s] = (s == 2) ? fmax(t[s], x[s]) : t[s] + x[s];
                }
                remaining &= ~__ballot(mine);
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < K * kSegStats; i += kSegBlock) out[i] = table[i];
    // out-of-range count of the workgroup (small integers: any order gives the same double)
    double o = oor;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) o += seg_shfl_xor(o, off);
    __shared__ double oor_wave[kSegBlock / 64];
    if (lane == 0) oor_wave[wave] = o;
    __syncthreads();
    double total = 0.0;
    for (int w = 0; w < kSegBlock / 64; ++w) total += oor_wave[w];
    __syncthreads();
    return total;
}

// Final sums over the workgroups' tables, by ONE workgroup of kSegBlock threads.  Slot (k, s) is
// summed by a group of T threads (T = the largest power of two with K * 7 * T <= kSegBlock, at
// least 1), each over the blocks b = j, j + T, ... in order, then the T partial sums in order.
__device__ __forceinline__ void seg_finalize(const SegStatsArgs& a, int64_t nblk, double* scratch /* [kSegBlock] */)
{
    const int tid = threadIdx.x;
    const int slots = a.K * kSegStats;
    int T = 1;
    while (slots * T * 2 <= kSegBlock) T *= 2;
    for (int base = 0; base < slots; base += kSegBlock / T) {
        const int slot = base + tid / T;
        const int j = tid % T;
        double acc = 0.0;
        const bool is_max = (slot % kSegStats) == 2;
        if (slot < slots && tid / T < kSegBlock / T) {
            for (int64_t b = j; b < nblk; b += T) {
                const double p = a.part[b * slots + slot];
                acc = is_max ? fmax(acc, p) : acc + p;
            }
        }
        __syncthreads();
        scratch[tid] = acc;
        __syncthreads();
        if (slot < slots && j == 0) {
            double s = scratch[tid];
            for (int q = 1; q < T; ++q) s = is_max ? fmax(s, scratch[tid + q]) : s + scratch[tid + q];
            const int k = slot / kSegStats;
            switch (slot % kSegStats) {
            case 0: a.count[k] = (int64_t)s; break;
            case 1: a.ratio_sum[k] = s; break;
            case 2: a.ratio_max[k] = (float)s; break;
            case 3: a.clipped[k] = (int64_t)s; break;
            case 4: a.kl_sum[k] = s; break;
            case 5: a.ent_sum[k] = s; break;
            default: a.masked[k] = (int64_t)s; break;
            }
        }
    }
    // out-of-range tokens
    double o = 0.0;
    for (int64_t b = tid; b < nblk; b += kSegBlock) o += a.part_oor[b];
    __syncthreads();
    scratch[tid] = o;
    __syncthreads();
    if (tid == 0 && a.out_of_range) {
        double s = 0.0;
        for (int q = 0; q < kSegBlock; ++q) s += scratch[q];
        *a.out_of_range = (int64_t)s;
    }
}

inline size_t seg_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline size_t seg_workspace_bytes(int64_t N, int32_t K)
{
    const size_t nblk = (size_t)((N + kSegBlock - 1) / kSegBlock);
    return seg_align_up(nblk * (size_t)K * kSegStats * sizeof(double), 256) + seg_align_up(nblk * sizeof(double), 256);
}

}  // namespace ulorl_detail

#endif
