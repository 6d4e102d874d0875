// Declarations shared by the translation units of libulorl (not part of the public ABI).
#ifndef ULORL_INTERNAL_HPP
#define ULORL_INTERNAL_HPP

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ulorl.h"

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
};

struct WorkspaceLayout {
    size_t slots, syncfail, hsum, rflags, part_sum, part_cnt, defer, badcu, total;
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
                          uint8_t* resp_gate, void* workspace, const WorkspaceLayout& wl);

// Enqueues response_entropy_kernel, token_terms_kernel and loss_finalize_kernel.
void launch_token_epilogue(const TokenArgs& a, const WorkspaceLayout& wl, float* loss, int64_t* counters,
                           hipStream_t st);

// Launch shapes, set with ulorl_tune().  Defaults from sweeps on 131072 x 151936 bf16 (logits
// path) and 32768 x 2048 x 151936 (lm_head variant).  The one-workgroup-per-row forward and fused
// kernels share one shape so that their row statistics are bit-identical, and so do the piece-wise
// forward and the row-cooperative kernel (the backward is elementwise, its shape does not change
// results).
struct Tuning {
    int fwd_threads = 512, fwd_unroll = 8;
    int bwd_threads = 256, bwd_unroll = 4;
    int fused_threads = 512, fused_unroll = 8;
    int gemm_tile = 7;     // index into the compiled-in GEMM tile shapes
    int bwd_oneshot = 1;   // standalone backward by one-shot 4 KB workgroups (0: one looping workgroup per row)
    int fused_cluster = 1; // one-call path by row-cooperative workgroups (0: one looping workgroup per row)
    int fwd_pieces = 1;    // forward statistics by pieces when a workspace is given (0: one looping workgroup per row)
    int fused_vpt = 0;     // 16-byte vectors per thread of the row-cooperative kernel (0: chosen from V)
    int sync_spins = 1 << 24;  // polls before a workgroup of the row-cooperative kernel gives up on its partners
};
Tuning& tuning();
constexpr int kGemmTileCount = 9;
inline int gemm_tile_choice() { return tuning().gemm_tile; }

}  // namespace ulorl_detail

#endif
