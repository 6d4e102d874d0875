// Launch-shape knobs of libulorl (process-wide; not thread safe against concurrent launches).
#include "ulorl_internal.hpp"

namespace ulorl_detail {
Tuning& tuning()
{
    static Tuning t;
    return t;
}
}  // namespace ulorl_detail

extern "C" int32_t ulorl_tune(int32_t knob, int32_t value)
{
    ulorl_detail::Tuning& t = ulorl_detail::tuning();
    const bool threads_ok = value == 256 || value == 512 || value == 1024;
    const bool unroll_ok = value == 2 || value == 4 || value == 8;
    switch (knob) {
    case ULORL_TUNE_FWD_THREADS: if (!threads_ok) return ULORL_ERR_PARAM; t.fwd_threads = value; return ULORL_OK;
    case ULORL_TUNE_FWD_UNROLL:  if (!unroll_ok) return ULORL_ERR_PARAM;  t.fwd_unroll = value;  return ULORL_OK;
    case ULORL_TUNE_BWD_THREADS: if (!threads_ok) return ULORL_ERR_PARAM; t.bwd_threads = value; return ULORL_OK;
    case ULORL_TUNE_BWD_UNROLL:  if (!unroll_ok) return ULORL_ERR_PARAM;  t.bwd_unroll = value;  return ULORL_OK;
    case ULORL_TUNE_FUSED_THREADS: if (!threads_ok) return ULORL_ERR_PARAM; t.fused_threads = value; return ULORL_OK;
    case ULORL_TUNE_FUSED_UNROLL:  if (!unroll_ok) return ULORL_ERR_PARAM;  t.fused_unroll = value;  return ULORL_OK;
    case ULORL_TUNE_BWD_ONESHOT: if (value != 0 && value != 1) return ULORL_ERR_PARAM; t.bwd_oneshot = value; return ULORL_OK;
    case ULORL_TUNE_FUSED_CLUSTER: if (value != 0 && value != 1) return ULORL_ERR_PARAM; t.fused_cluster = value; return ULORL_OK;
    case ULORL_TUNE_FWD_PIECES: if (value != 0 && value != 1) return ULORL_ERR_PARAM; t.fwd_pieces = value; return ULORL_OK;
    case ULORL_TUNE_FUSED_VPT:
        if (value != 0 && value != 4 && value != 8 && value != 10 && value != 12 && value != 15) return ULORL_ERR_PARAM;
        t.fused_vpt = value;
        return ULORL_OK;
    case ULORL_TUNE_SYNC_SPINS: if (value < 1) return ULORL_ERR_PARAM; t.sync_spins = value; return ULORL_OK;
    case ULORL_TUNE_GEMM_TILE:
        if (value < 0 || value >= ulorl_detail::kGemmTileCount) return ULORL_ERR_PARAM;
        t.gemm_tile = value;
        return ULORL_OK;
    default: return ULORL_ERR_PARAM;
    }
}
