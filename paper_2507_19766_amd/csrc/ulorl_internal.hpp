// Declarations shared by the translation units of libulorl (not part of the public ABI).
#ifndef ULORL_INTERNAL_HPP
#define ULORL_INTERNAL_HPP

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ulorl.h"
#include "segment_stats.hpp"

namespace ulorl_detail {

constexpr int kTokBlock = 1024;  // tokens per workgroup of the O(N) epilogue kernels

// Arguments of the O(N) epilogue (per-response entropy, token terms, loss reduction).
struct TokenArgs {
    const float* logp;
    const float* entropy;
    const float* lse;
    const int32_t* token_ids;
    const int32_t* cu;
    const int32_t* segment_ids;
    const float* old_logp;
    const float* adv;
    float* gcoef;
    uint8_t* mask;
    float* ratio;
    int32_t* seg_out;
    float* resp_entropy;
    uint8_t* resp_gate;
    const uint32_t* sync_fail;  // one word (may be NULL): a wait of the row-cooperative kernel expired
    double* hsum;       // [R] workspace
    uint32_t* rflags;   // [R] workspace
    double* part_sum;   // [nblk] workspace
    int64_t* part_cnt;  // [nblk * 4] workspace
    int64_t N;
    int32_t V, R;
    int32_t is_mode, gate_mode, seg_len;
    double eps_low, eps_high, tau, sigma, D;
    double log_tau, inv_D;   // ln(tau), 1 / D
    SegStatsArgs seg;        // per-segment diagnostics as a by-product (seg.K == 0: not wanted)
};

struct WorkspaceLayout {
    size_t slots, syncfail, hsum, rflags, part_sum, part_cnt, defer, badcu, zy, defer_list, defer_count, total;
    int64_t nblk;
};

struct ClusterShape {
    int vpt;      // 16-byte vectors per thread
    int pieces;   // workgroups per row (0: shape not supported)
};
ClusterShape cluster_shape(int64_t V, int32_t dt);

// V = 0: no exchange slots (callers that never run the row-cooperative kernel).
WorkspaceLayout workspace_layout(int64_t N, int64_t V, int32_t R);

// Host-side validation of the objective's scalar parameters and required pointers.
int32_t check_objective_args(const int32_t* cu_seqlens, int32_t R, const float* old_logp, const ulorl_params* p,
                             const float* loss, const float* gcoef);

TokenArgs make_token_args(int64_t N, int64_t V, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R,
                          const int32_t* segment_ids, const float* old_logp, const float* advantages,
                          const ulorl_params* p, float* logp, float* entropy, float* lse, float* gcoef,
                          uint8_t* mpt_mask, float* ratio, int32_t* segment_out, float* resp_entropy,
                          uint8_t* resp_gate, void* workspace, const WorkspaceLayout& wl, const SegStatsArgs& seg);

// Enqueues response_entropy_kernel, token_terms_kernel and loss_finalize_kernel.
void launch_token_epilogue(const TokenArgs& a, const WorkspaceLayout& wl, float* loss, int64_t* counters,
                           hipStream_t st);

// Launch options of one call, validated and with the defaults filled in.
struct LaunchOpts {
    bool per_row = false;         // ULORL_LAUNCH_PER_ROW
    bool dense_rows = false;      // ULORL_LAUNCH_DENSE_ROWS
    int sync_spins = 1 << 24;
    int gemm_tile = 0;
    int gemm_group_m = 4;
};
int32_t resolve_launch(const ulorl_launch* launch, LaunchOpts* out);

// Validates an optional ulorl_segment_stats against N and turns it into kernel arguments
// (out->K == 0 when st is NULL).
int32_t resolve_segment_stats(const ulorl_segment_stats* st, int64_t N, SegStatsArgs* out);

}  // namespace ulorl_detail

#endif
