// lm_head variant of the UloRL token loss for gfx950: logits = hidden . W are produced tile by
// tile on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) and consumed in registers;
// the [N, V] logits tensor never exists in memory.
//
// One tiled bf16 GEMM main loop, C[m, n] = sum_k A[m, k] * B[n, k] with BOTH operands contiguous
// along the contraction index, serves every product of the path:
//   forward   z^T[v, t] = Wt[v, :] . hidden[t, :]      epilogue: online softmax statistics per token
//   backward  z^T again                                 epilogue: dz = g (onehot - softmax), stored
//                                                        per vocabulary chunk as dZc[t, v] and dZc^T[v, t]
//             dHidden[t, k] += dZc[t, :] . W[k, chunk]   (fp32 accumulation across chunks)
//             dW[k, chunk]   = Ht[k, :] . dZc^T[v, :]    (each element written once)
// Wt = W^T and Ht = hidden^T are made once per call by a tiled transpose, so that no operand
// needs a transposing load.  In the z^T orientation a lane of the 32x32 MFMA result holds one
// token column and 16 vocabulary rows, which makes the softmax reductions lane-local.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <mutex>
#include <type_traits>
#include <unordered_map>

#include "ulorl.h"
#include "ulorl_internal.hpp"

using namespace ulorl_detail;

#pragma clang fp contract(off)

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kEmpty = -1.0e30f;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint16_t bf16_t;  // raw storage

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 x = {lo, hi};
    bf16x2 b = __builtin_convertvector(x, bf16x2);  // round to nearest even
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ bf16_t to_bf16(float x) { return (bf16_t)(pack_bf16x2(x, 0.0f) & 0xffffu); }

// ---------------------------------------------------------------------------------------------
// tiled GEMM main loop
// ---------------------------------------------------------------------------------------------
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, bool DIRECT_ = false, int WG_PER_CU_ = 1>
struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_;
    static constexpr bool DIRECT = DIRECT_;                // global -> LDS without passing through registers
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    // workgroups meant to share a compute unit; the register budget follows from it (waves per SIMD)
    static constexpr int WG_PER_CU = WG_PER_CU_;
    static constexpr int WAVES_PER_SIMD = (WG_PER_CU * WAVES_M * WAVES_N + 3) / 4;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int MB = WM / 32, NB = WN / 32;      // 32x32 result blocks per wave
    static constexpr int LDS_STRIDE = BK + 8;              // bf16 elements; the pad spreads rows over banks
    static constexpr int A_STAGE = BM * LDS_STRIDE;
    static constexpr int B_STAGE = BN * LDS_STRIDE;
    static constexpr int VEC_PER_ROW = BK / 8;
    static constexpr int A_VECS = BM * VEC_PER_ROW / NT;   // 16-byte vectors each thread moves per stage
    static constexpr int B_VECS = BN * VEC_PER_ROW / NT;
    static constexpr size_t LDS_BYTES = 2 * (size_t)(A_STAGE + B_STAGE) * sizeof(bf16_t);
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile shape");
    static_assert(!DIRECT || (BK == 64 && BM % (8 * (NT / 64)) == 0 && BN % (8 * (NT / 64)) == 0),
                  "direct-to-LDS tile shape");
    static_assert(LDS_BYTES * WG_PER_CU <= 160 * 1024, "LDS per compute unit");
    static_assert((BM * VEC_PER_ROW) % NT == 0 && (BN * VEC_PER_ROW) % NT == 0, "load split");
};

// acc[bi][bj][r] holds C[m, n] with
//   m = m0 + wave_m*WM + bi*32 + 8*(r/4) + 4*(lane/32) + (r%4),   n = n0 + wave_n*WN + bj*32 + lane%32.
// Rows beyond M / N are computed from clamped addresses and must be ignored by the caller;
// contraction indices beyond K contribute zero.  K and the leading dimensions are multiples of 8.
template <class Cfg>
__device__ __forceinline__ void gemm_tn_mainloop(const bf16_t* __restrict__ A, int64_t lda, int M, int m0,
                                                 const bf16_t* __restrict__ B, int64_t ldb, int N, int n0, int K,
                                                 f32x16 (&acc)[Cfg::MB][Cfg::NB], bf16_t* lds)
{
    constexpr int NT = Cfg::NT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave / Cfg::WAVES_N;
    const int wave_n = wave % Cfg::WAVES_N;
    bf16_t* sA = lds;
    bf16_t* sB = lds + 2 * Cfg::A_STAGE;

#pragma unroll
    for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.0f;

    // Per-thread sources of this tile: a workgroup-uniform base (kept in scalar registers and
    // advanced along K) plus a 32-bit byte offset per vector (rows clamped into range), so the
    // hot loop carries no 64-bit vector address arithmetic.
    const char* a_tile = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
    const char* b_tile = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
    uint32_t oa[Cfg::A_VECS], ob[Cfg::B_VECS];
    int ka[Cfg::A_VECS], kb[Cfg::B_VECS];
    int la[Cfg::A_VECS], lb[Cfg::B_VECS];
#pragma unroll
    for (int i = 0; i < Cfg::A_VECS; ++i) {
        const int idx = tid + i * NT;
        const int row = idx / Cfg::VEC_PER_ROW, kv = idx % Cfg::VEC_PER_ROW;
        const int gr = (m0 + row < M) ? row : (M - 1 - m0);
        oa[i] = (uint32_t)(((int64_t)gr * lda + kv * 8) * 2);
        ka[i] = kv * 8;
        la[i] = row * Cfg::LDS_STRIDE + kv * 8;
    }
#pragma unroll
    for (int i = 0; i < Cfg::B_VECS; ++i) {
        const int idx = tid + i * NT;
        const int row = idx / Cfg::VEC_PER_ROW, kv = idx % Cfg::VEC_PER_ROW;
        const int gr = (n0 + row < N) ? row : (N - 1 - n0);
        ob[i] = (uint32_t)(((int64_t)gr * ldb + kv * 8) * 2);
        kb[i] = kv * 8;
        lb[i] = row * Cfg::LDS_STRIDE + kv * 8;
    }

    u32x4 ra[Cfg::A_VECS], rb[Cfg::B_VECS];
    const u32x4 zero = {0u, 0u, 0u, 0u};
    auto fetch_full = [&](int k0) {      // whole tile inside the contraction range
        const char* pa = a_tile + (int64_t)k0 * 2;
        const char* pb = b_tile + (int64_t)k0 * 2;
#pragma unroll
        for (int i = 0; i < Cfg::A_VECS; ++i) ra[i] = *reinterpret_cast<const u32x4*>(pa + oa[i]);
#pragma unroll
        for (int i = 0; i < Cfg::B_VECS; ++i) rb[i] = *reinterpret_cast<const u32x4*>(pb + ob[i]);
    };
    auto fetch_ragged = [&](int k0) {    // last tile: vectors past K contribute zero
        const char* pa = a_tile + (int64_t)k0 * 2;
        const char* pb = b_tile + (int64_t)k0 * 2;
#pragma unroll
        for (int i = 0; i < Cfg::A_VECS; ++i)
            ra[i] = (k0 + ka[i] < K) ? *reinterpret_cast<const u32x4*>(pa + oa[i]) : zero;
#pragma unroll
        for (int i = 0; i < Cfg::B_VECS; ++i)
            rb[i] = (k0 + kb[i] < K) ? *reinterpret_cast<const u32x4*>(pb + ob[i]) : zero;
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int i = 0; i < Cfg::A_VECS; ++i)
            *reinterpret_cast<u32x4*>(sA + stage * Cfg::A_STAGE + la[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < Cfg::B_VECS; ++i)
            *reinterpret_cast<u32x4*>(sB + stage * Cfg::B_STAGE + lb[i]) = rb[i];
    };

    const int frag_row = lane & 31;
    const int frag_k = 8 * (lane >> 5);
    const int a_base = (wave_m * Cfg::WM + frag_row) * Cfg::LDS_STRIDE + frag_k;
    const int b_base = (wave_n * Cfg::WN + frag_row) * Cfg::LDS_STRIDE + frag_k;
    auto compute = [&](int cur) {
        const bf16_t* cA = sA + cur * Cfg::A_STAGE + a_base;
        const bf16_t* cB = sB + cur * Cfg::B_STAGE + b_base;
#pragma unroll
        for (int kk = 0; kk < Cfg::BK / 16; ++kk) {
            bf16x8 fa[Cfg::MB], fb[Cfg::NB];
#pragma unroll
            for (int bi = 0; bi < Cfg::MB; ++bi)
                fa[bi] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(cA + bi * 32 * Cfg::LDS_STRIDE + kk * 16));
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj)
                fb[bj] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(cB + bj * 32 * Cfg::LDS_STRIDE + kk * 16));
#pragma unroll
            for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
                for (int bj = 0; bj < Cfg::NB; ++bj)
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[bi], fb[bj], acc[bi][bj], 0, 0, 0);
        }
    };

    // Double-buffered pipeline, one barrier per K tile: the global loads of tile kt+1 are in
    // flight while tile kt is multiplied out of LDS.  The hot loop runs over the tiles that lie
    // wholly inside K and has no conditional code; a ragged last tile is peeled off.
    const int KT = (K + Cfg::BK - 1) / Cfg::BK;
    const int KT_full = K / Cfg::BK;
    if (KT_full > 0) fetch_full(0); else fetch_ragged(0);
    stash(0);
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < KT_full; ++kt) {
        fetch_full((kt + 1) * Cfg::BK);
        __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of the multiply: its latency hides there
        compute(kt & 1);
        stash((kt + 1) & 1);
        __syncthreads();
    }
    for (; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) fetch_ragged((kt + 1) * Cfg::BK);
        compute(kt & 1);
        if (more) stash((kt + 1) & 1);
        __syncthreads();
    }
}

// Scheduling request for one MFMA step of the direct main loop: the first MFMA, READS LDS reads,
// COPIES x (one global -> LDS copy, one MFMA), the remaining MFMAs.
template <int COPIES, int READS, int MFMAS>
__device__ __forceinline__ void step_pattern()
{
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
#pragma unroll
    for (int i = 0; i < COPIES; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, MFMAS - 1 - COPIES, 0);
}

// Word 3 of a raw (unstructured, stride 0) buffer descriptor on gfx9-family parts: 32-bit data format.
constexpr int kRawBufferFlags = 0x00020000;
// A tile's rows are addressed by 32-bit byte offsets from its first row: 256 rows of at most this
// many bf16 elements stay below 2^31 bytes.
constexpr int64_t kMaxLeadingDim = 1 << 22;

// The same product with the tiles copied global -> LDS by the load unit itself
// (buffer_load_dwordx4 ... lds: lane L of a wave deposits its 16 bytes at lds_base + 16 L), so the
// staging registers, the ds_write instructions and the wait between a load's return and its
// write disappear from the loop.  A wave-instruction fills 64 consecutive 16-byte slots = 8 rows
// of a BK = 64 tile or 16 rows of a BK = 32 tile; rows are therefore unpadded, and bank conflicts
// are avoided by storing vector kv of row r in slot (kv xor swz(r)) of that row (each lane simply
// fetches from global the vector that belongs in its slot).  A fragment read (ds_read_b128) is
// served 16 lanes = 16 consecutive tile rows = 256 bytes per clock, so those 16 rows must land in
// 16 different 16-byte columns of the 256-byte bank line: swz(r) = (r / 2) mod 8 for 128-byte
// rows, (r / 4) mod 4 for 64-byte rows.  Needs K to be a multiple of BK.
template <class Cfg>
__device__ __forceinline__ void gemm_tn_mainloop_direct(const bf16_t* __restrict__ A, int64_t lda, int M, int m0,
                                                        const bf16_t* __restrict__ B, int64_t ldb, int N, int n0, int K,
                                                        f32x16 (&acc)[Cfg::MB][Cfg::NB], bf16_t* lds)
{
    constexpr int NW = Cfg::NT / 64;
    constexpr int BK = Cfg::BK;
    constexpr int VPR = BK / 8;                   // 16-byte vectors per tile row
    constexpr int RPI = 64 / VPR;                 // tile rows one wave-instruction fills
    constexpr int A_INSTR = Cfg::BM / RPI / NW;   // wave-instructions per stage and operand
    constexpr int B_INSTR = Cfg::BN / RPI / NW;
    constexpr int A_STAGE = Cfg::BM * BK, B_STAGE = Cfg::BN * BK;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave / Cfg::WAVES_N;
    const int wave_n = wave % Cfg::WAVES_N;
    bf16_t* sA = lds;
    bf16_t* sB = lds + 2 * A_STAGE;

#pragma unroll
    for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.0f;

    const char* a_tile = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
    const char* b_tile = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
    // this lane's source for wave-instruction j: row (j*NW + wave)*RPI + lane/VPR, vector (lane%VPR) xor swz(row)
    auto swz = [](int row) { return VPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    const int sub_row = lane / VPR;
    uint32_t oa[A_INSTR], ob[B_INSTR];
#pragma unroll
    for (int j = 0; j < A_INSTR; ++j) {
        const int row = (j * NW + wave) * RPI + sub_row;
        const int kv = (lane % VPR) ^ swz(row);
        const int gr = (m0 + row < M) ? row : (M - 1 - m0);
        oa[j] = (uint32_t)(((int64_t)gr * lda + kv * 8) * 2);
    }
#pragma unroll
    for (int j = 0; j < B_INSTR; ++j) {
        const int row = (j * NW + wave) * RPI + sub_row;
        const int kv = (lane % VPR) ^ swz(row);
        const int gr = (n0 + row < N) ? row : (N - 1 - n0);
        ob[j] = (uint32_t)(((int64_t)gr * ldb + kv * 8) * 2);
    }
    // The copies are buffer loads: a descriptor per operand slab (base = first row of the tile,
    // extent = up to the end of its last valid row) in scalar registers, the lane's 32-bit byte
    // offset, and the K position as the scalar offset.  No 64-bit address arithmetic is left in
    // the loop, and the hardware drops any access beyond the extent instead of faulting.
    const int rows_a = min(Cfg::BM, M - m0), rows_b = min(Cfg::BN, N - n0);
    const uint64_t extent_a = ((uint64_t)(rows_a - 1) * (uint64_t)lda + (uint64_t)K) * 2;
    const uint64_t extent_b = ((uint64_t)(rows_b - 1) * (uint64_t)ldb + (uint64_t)K) * 2;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(a_tile), 0, (int)(uint32_t)min(extent_a, (uint64_t)0xffffffffu), kRawBufferFlags);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(b_tile), 0, (int)(uint32_t)min(extent_b, (uint64_t)0xffffffffu), kRawBufferFlags);
    auto fetch_a = [&](int k0, int stage) {
#pragma unroll
        for (int j = 0; j < A_INSTR; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a,
                                                     (__attribute__((address_space(3))) void*)(sA + stage * A_STAGE + (j * NW + wave) * RPI * BK),
                                                     16, oa[j], k0 * 2, 0, 0);
    };
    auto fetch_b = [&](int k0, int stage) {
#pragma unroll
        for (int j = 0; j < B_INSTR; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b,
                                                     (__attribute__((address_space(3))) void*)(sB + stage * B_STAGE + (j * NW + wave) * RPI * BK),
                                                     16, ob[j], k0 * 2, 0, 0);
    };

    // fragment sources: row = tile row of this lane, vector kg = 2 kk + lane/32, stored at slot kg xor swz(row)
    const int frag_row = lane & 31;
    const int a_row = (wave_m * Cfg::WM + frag_row) * BK;
    const int b_row = (wave_n * Cfg::WN + frag_row) * BK;
    const int frag_swz = swz(frag_row);            // wave and block offsets are multiples of 32 rows: no effect on swz
    int koff[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) koff[kk] = (((2 * kk + (lane >> 5)) ^ frag_swz) * 8);
    constexpr int KK = BK / 16;                   // MFMA steps per K tile (even)
    bf16x8 fa[2][Cfg::MB], fb[2][Cfg::NB];        // two fragment sets: one feeds the MFMAs while the other loads
    // read order = the order in which the MFMAs first need the fragments (A0, B0.., A1..)
    auto load_frags = [&](int set, int stage, int kk) {
        const bf16_t* cA = sA + stage * A_STAGE + a_row + koff[kk];
        const bf16_t* cB = sB + stage * B_STAGE + b_row + koff[kk];
        fa[set][0] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(cA));
#pragma unroll
        for (int bj = 0; bj < Cfg::NB; ++bj)
            fb[set][bj] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(cB + bj * 32 * BK));
#pragma unroll
        for (int bi = 1; bi < Cfg::MB; ++bi)
            fa[set][bi] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(cA + bi * 32 * BK));
    };
    auto multiply = [&](int set) {
#pragma unroll
        for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj)
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][bi], fb[set][bj], acc[bi][bj], 0, 0, 0);
    };
    // Wanted order inside an MFMA step: the first MFMA (it carries the wait for this step's
    // fragments), then all LDS reads of the next step's fragments, then the other MFMAs.  A read
    // issued before that wait would be waited for as well: while global -> LDS copies are in
    // flight the compiler only emits full waits on the LDS counter.  A step that also issues
    // `copies` global -> LDS copies gets them one per MFMA: the address unit of the compute unit
    // takes 16 clocks per copy instruction and is shared by all waves, and a wave whose copy is
    // queued behind the others' cannot issue the MFMAs that follow it.
    static_assert(A_INSTR < Cfg::MB * Cfg::NB && B_INSTR < Cfg::MB * Cfg::NB, "copies per step");

    // Software pipeline over two LDS stages; tile kt lives in stage kt & 1.  Fragments of MFMA
    // step kk+1 are read from LDS while step kk multiplies.  The barrier that ends K tile kt sits
    // before its last step: by then every wave has read all it needs from that stage (its last
    // fragments are in registers), so after the barrier the copy of tile kt+2 may overwrite the
    // stage and the first fragments of tile kt+1 can be read, both underneath the last step's
    // MFMAs.  The A half of tile kt+2 is copied during that last step, the B half during the
    // first step of tile kt+1.
    const int KT = K / BK;
    static_assert(KK % 2 == 0 && KK >= 4, "the fragment sets alternate per MFMA step; first and last steps carry the copies");
    fetch_a(0, 0);
    fetch_b(0, 0);
    __builtin_amdgcn_s_waitcnt(0);     // the tile has landed in LDS (vmcnt) ...
    __syncthreads();                   // ... for every wave
    if (KT > 1) fetch_a(BK, 1);
    load_frags(0, 0, 0);
    auto mid_steps = [&](int cur) {    // MFMA steps 1 .. KK-2 of a K tile, then the barrier
#pragma unroll
        for (int kk = 1; kk + 1 < KK; ++kk) {
            load_frags((kk + 1) & 1, cur, kk + 1);
            multiply(kk & 1);
            step_pattern<0, Cfg::MB + Cfg::NB, Cfg::MB * Cfg::NB>();
        }
        __builtin_amdgcn_sched_barrier(0);  // the MFMAs above stay above: they run while the wave waits below
        __builtin_amdgcn_s_waitcnt(0);      // the next tile has landed (vmcnt), own LDS reads are done (lgkmcnt)
        __syncthreads();
    };
    int kt = 0;
    for (; kt + 2 < KT; ++kt) {            // steady state, free of conditional code
        const int cur = kt & 1;
        load_frags(1, cur, 1);
        fetch_b((kt + 1) * BK, cur ^ 1);
        multiply(0);
        step_pattern<B_INSTR, Cfg::MB + Cfg::NB, Cfg::MB * Cfg::NB>();
        mid_steps(cur);
        load_frags(0, cur ^ 1, 0);
        fetch_a((kt + 2) * BK, cur);
        multiply((KK - 1) & 1);
        step_pattern<A_INSTR, Cfg::MB + Cfg::NB, Cfg::MB * Cfg::NB>();
    }
    if (kt + 1 < KT) {                     // last but one tile: only the B half of the last tile is left to copy
        const int cur = kt & 1;
        load_frags(1, cur, 1);
        fetch_b((kt + 1) * BK, cur ^ 1);
        multiply(0);
        step_pattern<B_INSTR, Cfg::MB + Cfg::NB, Cfg::MB * Cfg::NB>();
        mid_steps(cur);
        load_frags(0, cur ^ 1, 0);
        multiply((KK - 1) & 1);
        step_pattern<0, Cfg::MB + Cfg::NB, Cfg::MB * Cfg::NB>();
        ++kt;
    }
    {                                      // last tile
        const int cur = kt & 1;
        load_frags(1, cur, 1);
        multiply(0);
        step_pattern<0, Cfg::MB + Cfg::NB, Cfg::MB * Cfg::NB>();
        mid_steps(cur);                    // its barrier: every wave is past its last LDS read, the caller may reuse LDS
        multiply((KK - 1) & 1);
    }
}

template <class Cfg>
__device__ __forceinline__ void gemm_tn_tile(const bf16_t* __restrict__ A, int64_t lda, int M, int m0,
                                             const bf16_t* __restrict__ B, int64_t ldb, int N, int n0, int K,
                                             f32x16 (&acc)[Cfg::MB][Cfg::NB], bf16_t* lds)
{
    if (K <= 0) {           // empty contraction (no live row): the product is zero
#pragma unroll
        for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.0f;
        __syncthreads();
        return;
    }
    if constexpr (Cfg::DIRECT) {
        if (K % Cfg::BK == 0) {
            gemm_tn_mainloop_direct<Cfg>(A, lda, M, m0, B, ldb, N, n0, K, acc, lds);
            return;
        }
    }
    gemm_tn_mainloop<Cfg>(A, lda, M, m0, B, ldb, N, n0, K, acc, lds);
}

// Workgroup -> tile mapping.  The hardware deals consecutive workgroup ids round-robin to the 8
// XCDs, each with its own L2.  Ids are first regrouped so that every XCD owns one contiguous
// range of logical tile numbers, and logical numbers walk the tile grid in blocks of group_m
// (default 4) tiles along M by all tiles along N (column-major inside the block): the 32
// workgroups resident on an XCD then cover about 4 x 8 tiles and share their A and B slices
// through that XCD's L2.
constexpr int kXcds = 8;

// bid: the workgroup's id within its kernel, or within its part of a launch that several products
// share (a part starts at a multiple of 8 workgroups, so bid % 8 is still the XCD).
__device__ __forceinline__ bool tile_coords(int bid, int num_m, int num_n, int group_m, int& tile_m, int& tile_n)
{
    const int total = num_m * num_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const int logical = (bid % kXcds) * per_xcd + bid / kXcds;
    if (bid / kXcds >= per_xcd || logical >= total) return false;
    const int group_size = group_m * num_n;
    const int group = logical / group_size;
    const int first_m = group * group_m;
    const int gm = min(group_m, num_m - first_m);
    const int in_group = logical % group_size;
    tile_m = first_m + in_group % gm;
    tile_n = in_group / gm;
    return true;
}

__host__ __device__ inline unsigned tile_grid(int num_m, int num_n)
{
    const int total = num_m * num_n;
    return (unsigned)(((total + kXcds - 1) / kXcds) * kXcds);
}

// ---------------------------------------------------------------------------------------------
// plain GEMM kernels: C = A . B^T with three ways of storing C
// ---------------------------------------------------------------------------------------------
enum { STORE_F32 = 0, STORE_F32_ACCUM = 1, STORE_BF16 = 2 };

// Writes a wave's result tile to row-major C with 16-byte accesses.  In the MFMA result layout a
// lane owns one column and 16 rows of a 32 x 32 block, so direct stores are 4 (or 2) bytes per lane;
// instead each 32-row slab of the wave tile goes through the wave's share of LDS (the main loop's
// stages, free by now) and is read back row-wise, one 16-byte vector per lane.  C must be 16-byte
// aligned with a row pitch that is a multiple of 16 bytes.  Every wave of the workgroup must call.
template <class Cfg, int STORE>
__device__ __forceinline__ void store_wave_tile_rows(const f32x16 (&acc)[Cfg::MB][Cfg::NB], void* __restrict__ C,
                                                     int64_t ldc, int M, int N, int m_wave, int n_wave,
                                                     unsigned char* lds_raw)
{
    constexpr int EB = STORE == STORE_BF16 ? 2 : 4;          // bytes per element of C
    constexpr int EPV = 16 / EB;                             // elements per 16-byte vector
    constexpr int ROW_BYTES = Cfg::WN * EB;
    constexpr int STRIDE = ROW_BYTES + 16;                   // padded: the four rows a lane pair writes fall in different banks
    constexpr int VPR = ROW_BYTES / 16;                      // vectors per slab row
    constexpr int RPI = 64 / VPR;                            // slab rows one wave-wide read covers
    static_assert(VPR <= 64 && 32 % RPI == 0, "slab shape");
    static_assert((size_t)32 * STRIDE <= Cfg::LDS_BYTES / (Cfg::NT / 64), "slab fits the wave's share of LDS");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char* slab = lds_raw + (size_t)wave * (Cfg::LDS_BYTES / (Cfg::NT / 64));
#pragma unroll
    for (int bi = 0; bi < Cfg::MB; ++bi) {
#pragma unroll
        for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int col = bj * 32 + (lane & 31);
                if (STORE == STORE_BF16) *reinterpret_cast<bf16_t*>(slab + row * STRIDE + col * 2) = to_bf16(acc[bi][bj][r]);
                else *reinterpret_cast<float*>(slab + row * STRIDE + col * 4) = acc[bi][bj][r];
            }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = i * RPI + lane / VPR;
            const int vec = lane % VPR;
            const u32x4 v = *reinterpret_cast<const u32x4*>(slab + row * STRIDE + vec * 16);
            const int m = m_wave + bi * 32 + row;
            const int n = n_wave + vec * EPV;
            if (m < M && n < N) {
                char* dst = reinterpret_cast<char*>(C) + ((int64_t)m * ldc + n) * EB;
                if (n + EPV <= N) {
                    if (STORE == STORE_F32_ACCUM) {
                        const f32x4 old = *reinterpret_cast<const f32x4*>(dst);
                        const f32x4 add = __builtin_bit_cast(f32x4, v);
                        *reinterpret_cast<f32x4*>(dst) = old + add;
                    } else {
                        *reinterpret_cast<u32x4*>(dst) = v;
                    }
                } else {                                     // ragged right edge: element by element
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        if (n + e >= N) break;
                        if (STORE == STORE_BF16) {
                            const uint32_t pair = v[e / 2];
                            reinterpret_cast<bf16_t*>(dst)[e] = (bf16_t)((e & 1) ? (pair >> 16) : (pair & 0xffffu));
                        } else {
                            const float x = __builtin_bit_cast(float, (uint32_t)v[e]);
                            if (STORE == STORE_F32_ACCUM) reinterpret_cast<float*>(dst)[e] += x;
                            else reinterpret_cast<float*>(dst)[e] = x;
                        }
                    }
                }
            }
        }
        __syncthreads();
    }
}

// One product C = A . B^T (A [M, K], B [N, K], both with K contiguous).  wide_rows: C allows
// 16-byte accesses.
struct GemmArgs {
    const bf16_t* A; int64_t lda; int M;
    const bf16_t* B; int64_t ldb; int N;
    int K;
    void* C; int64_t ldc;
    int wide_rows;
};

// The tile of workgroup `bid` (see tile_coords) of one product; workgroups beyond the tile grid
// return at once.
template <class Cfg, int STORE>
__device__ __forceinline__ void gemm_tn_block(int bid, const bf16_t* __restrict__ A, int64_t lda, int M,
                                              const bf16_t* __restrict__ B, int64_t ldb, int N, int K, void* __restrict__ C,
                                              int64_t ldc, int wide_rows, int group_m, unsigned char* lds_raw)
{
    bf16_t* lds = reinterpret_cast<bf16_t*>(lds_raw);
    if (M <= 0) return;
    int tile_m, tile_n;
    if (!tile_coords(bid, (M + Cfg::BM - 1) / Cfg::BM, (N + Cfg::BN - 1) / Cfg::BN, group_m, tile_m, tile_n)) return;
    const int m0 = tile_m * Cfg::BM, n0 = tile_n * Cfg::BN;
    f32x16 acc[Cfg::MB][Cfg::NB];
    gemm_tn_tile<Cfg>(A, lda, M, m0, B, ldb, N, n0, K, acc, lds);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
    if (wide_rows) {            // C allows 16-byte accesses (uniform over the grid)
        store_wave_tile_rows<Cfg, STORE>(acc, C, ldc, M, N, m0 + wm * Cfg::WM, n0 + wn * Cfg::WN, lds_raw);
        return;
    }
#pragma unroll
    for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < Cfg::NB; ++bj) {
            const int n = n0 + wn * Cfg::WN + bj * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * Cfg::WM + bi * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M && n < N) {
                    const int64_t off = (int64_t)m * ldc + n;
                    if (STORE == STORE_F32) ((float*)C)[off] = acc[bi][bj][r];
                    if (STORE == STORE_F32_ACCUM) ((float*)C)[off] += acc[bi][bj][r];
                    if (STORE == STORE_BF16) ((bf16_t*)C)[off] = to_bf16(acc[bi][bj][r]);
                }
            }
        }
}

template <class Cfg, int STORE>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WAVES_PER_SIMD, Cfg::WAVES_PER_SIMD)))
void gemm_tn_kernel(const GemmArgs g, int group_m)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    gemm_tn_block<Cfg, STORE>((int)blockIdx.x, g.A, g.lda, g.M, g.B, g.ldb, g.N, g.K, g.C, g.ldc, g.wide_rows, group_m, lds_raw);
}

// dst[c, r] = src[r, c] (bf16), 64x64 tiles through LDS, 16-byte accesses on both sides; columns
// of dst beyond `rows` up to dst_cols are written as zero (padding of the contraction dimension).
// cols, dst_cols and both leading dimensions are multiples of 8 and the bases 16-byte aligned.
// With a row map, row r of the source is src[row_map[r]] and the row count comes from the device
// (*dyn_rows): the gathered transpose of the live rows.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t* __restrict__ src, int64_t lds_, int rows,
                                                            int cols, bf16_t* __restrict__ dst, int64_t ldd,
                                                            int dst_cols, const int* __restrict__ row_map,
                                                            const int* __restrict__ dyn_rows)
{
    constexpr int P = 72;                       // row pitch in elements: 16-byte aligned rows, spread over the banks
    __shared__ __attribute__((aligned(16))) bf16_t tile[64 * P];
    if (dyn_rows != nullptr) rows = min(rows, *dyn_rows);
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int idx = (int)threadIdx.x + 256 * j;
        const int i = idx >> 3, vec = idx & 7;
        const int r = r0 + i, c = c0 + vec * 8;
        u32x4 x = {0u, 0u, 0u, 0u};
        if (r < rows && c < cols)
            x = *reinterpret_cast<const u32x4*>(src + (int64_t)(row_map != nullptr ? row_map[r] : r) * lds_ + c);
        *reinterpret_cast<u32x4*>(tile + i * P + vec * 8) = x;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int idx = (int)threadIdx.x + 256 * j;
        const int ci = idx >> 3, rv = idx & 7;
        const int c = c0 + ci, r = r0 + rv * 8;
        if (c < cols && r < dst_cols) {
            u32x4 x;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                x[q] = (uint32_t)tile[(rv * 8 + 2 * q) * P + ci] | ((uint32_t)tile[(rv * 8 + 2 * q + 1) * P + ci] << 16);
            *reinterpret_cast<u32x4*>(dst + (int64_t)c * ldd + r) = x;
        }
    }
}

// d_hidden[t, :] = bf16(acc[pos[t], :]) (pos == NULL: acc[t, :]); rows without a live position are zero.
// One thread converts 8 elements (Hd is a multiple of 8; both buffers 16-byte aligned).
__global__ void dhidden_finish_kernel(const float* __restrict__ acc, const int* __restrict__ pos, int64_t N, int Hd,
                                      bf16_t* __restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int vpr = Hd / 8;
    const int64_t t = i / vpr;
    if (t >= N) return;
    const int c = (int)(i - t * vpr) * 8;
    const int64_t j = pos != nullptr ? (int64_t)pos[t] : t;
    u32x4 out = {0u, 0u, 0u, 0u};
    if (j >= 0) {
        const u32x4 lo = *reinterpret_cast<const u32x4*>(acc + j * Hd + c);
        const u32x4 hi = *reinterpret_cast<const u32x4*>(acc + j * Hd + c + 4);
        out[0] = pack_bf16x2(__builtin_bit_cast(float, (uint32_t)lo[0]), __builtin_bit_cast(float, (uint32_t)lo[1]));
        out[1] = pack_bf16x2(__builtin_bit_cast(float, (uint32_t)lo[2]), __builtin_bit_cast(float, (uint32_t)lo[3]));
        out[2] = pack_bf16x2(__builtin_bit_cast(float, (uint32_t)hi[0]), __builtin_bit_cast(float, (uint32_t)hi[1]));
        out[3] = pack_bf16x2(__builtin_bit_cast(float, (uint32_t)hi[2]), __builtin_bit_cast(float, (uint32_t)hi[3]));
    }
    *reinterpret_cast<u32x4*>(dst + t * Hd + c) = out;
}

// ---------------------------------------------------------------------------------------------
// live rows of the backward pass
// ---------------------------------------------------------------------------------------------
// A token whose coefficient is zero (masked as a well-mastered positive token, on the clipped
// branch, zero advantage, or flagged) contributes nothing to d_W and has a zero d_hidden row.  The
// backward pass therefore runs its three products over the LIVE rows only: their indices are
// collected in order (so that every sum keeps a fixed order), hidden is gathered, and the kernels
// take the live count from device memory.  The dynamic mask of the method makes this count
// much smaller than N whenever many positive tokens are mastered.
constexpr int kLiveBlock = 1024;

__device__ __forceinline__ bool row_has_gradient(float g, float l, int32_t y, int32_t V)
{
    return (g != 0.0f) && (fabsf(g) <= 3.0e38f) && (fabsf(l) <= 3.0e38f) && y >= 0 && y < V;
}

// Inclusive prefix sum over a workgroup of kLiveBlock threads; *total = the workgroup's sum.
__device__ __forceinline__ int live_block_scan(int v, int* wave_tot, int* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(v, off);
        if (lane >= off) v += up;
    }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = v;
    __syncthreads();
    int before = 0, all = 0;
    for (int w = 0; w < kLiveBlock / 64; ++w) {
        const int x = wave_tot[w];
        before += w < wave ? x : 0;
        all += x;
    }
    *total = all;
    return v + before;
}

__global__ __launch_bounds__(kLiveBlock) void live_count_kernel(const float* __restrict__ gcoef, const float* __restrict__ lse,
                                                                const int32_t* __restrict__ token_ids, float grad_out,
                                                                int64_t N, int32_t V, int* __restrict__ block_count)
{
    __shared__ int wave_tot[kLiveBlock / 64];
    const int64_t t = (int64_t)blockIdx.x * kLiveBlock + threadIdx.x;
    const int live = t < N && row_has_gradient(gcoef[t] * grad_out, lse[t], token_ids[t], V);
    int total;
    live_block_scan(live, wave_tot, &total);
    if (threadIdx.x == 0) block_count[blockIdx.x] = total;
}

// One workgroup: exclusive prefix sums of the blocks' counts (in place) and the total.
__global__ __launch_bounds__(kLiveBlock) void live_scan_kernel(int* __restrict__ block_count, int nblk, int* __restrict__ n_live)
{
    __shared__ int wave_tot[kLiveBlock / 64];
    int base = 0;
    for (int b0 = 0; b0 < nblk; b0 += kLiveBlock) {
        const int b = b0 + threadIdx.x;
        const int c = b < nblk ? block_count[b] : 0;
        int total;
        const int incl = live_block_scan(c, wave_tot, &total);
        if (b < nblk) block_count[b] = base + incl - c;
        base += total;
    }
    if (threadIdx.x == 0) *n_live = base;
}

// pos[t] = position of row t among the live rows (-1: not live); row_map[position] = t.
__global__ __launch_bounds__(kLiveBlock) void live_fill_kernel(const float* __restrict__ gcoef, const float* __restrict__ lse,
                                                               const int32_t* __restrict__ token_ids, float grad_out,
                                                               int64_t N, int32_t V, const int* __restrict__ block_offset,
                                                               int* __restrict__ pos, int* __restrict__ row_map)
{
    __shared__ int wave_tot[kLiveBlock / 64];
    const int64_t t = (int64_t)blockIdx.x * kLiveBlock + threadIdx.x;
    const int live = t < N && row_has_gradient(gcoef[t] * grad_out, lse[t], token_ids[t], V);
    int total;
    const int incl = live_block_scan(live, wave_tot, &total);
    if (t < N) {
        const int p = block_offset[blockIdx.x] + incl - 1;
        pos[t] = live ? p : -1;
        if (live) row_map[p] = (int)t;
    }
}

// dst[j, :] = src[row_map[j], :] for j < *n_live (16-byte vectors; cols is a multiple of 8).
__global__ void gather_rows_kernel(const bf16_t* __restrict__ src, int cols, const int* __restrict__ row_map,
                                   const int* __restrict__ n_live, int64_t N, bf16_t* __restrict__ dst)
{
    const int vpr = cols / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t j = i / vpr;
    if (j >= N || j >= *n_live) return;
    const int v = (int)(i - j * vpr);
    reinterpret_cast<u32x4*>(dst + j * cols)[v] = reinterpret_cast<const u32x4*>(src + (int64_t)row_map[j] * cols)[v];
}

// n4 vectors of four floats (the accumulator's size is a multiple of 8 elements, its base 256-byte aligned)
__global__ void fill_zero_f32_kernel(float* p, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) reinterpret_cast<u32x4*>(p)[i] = u32x4{0u, 0u, 0u, 0u};
}

// ---------------------------------------------------------------------------------------------
// forward: softmax statistics from z^T tiles
// ---------------------------------------------------------------------------------------------
// (m, S, T) with T = sum e^(z-m) (z-m) in natural units; exact when the maxima coincide.
__device__ __forceinline__ void merge_nat(float& m, float& S, float& T, float m2, float S2, float T2)
{
    const float M = fmaxf(m, m2);
    const float d1 = m - M, d2 = m2 - M;
    const float s1 = fast_exp2(d1 * kLog2e), s2 = fast_exp2(d2 * kLog2e);
    T = s1 * fmaf(d1, S, T) + s2 * fmaf(d2, S2, T2);
    S = s1 * S + s2 * S2;
    m = M;
}

// Partial statistics of token t over one slice of the vocabulary: (max, sum, weighted sum,
// chosen logit or kEmpty).
struct StatQuad {
    float m, S, T, zy;
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WAVES_PER_SIMD, Cfg::WAVES_PER_SIMD)))
void lmhead_stats_kernel(const bf16_t* __restrict__ Wt, const bf16_t* __restrict__ H, int Hd, int V, int Ntok,
                         const int32_t* __restrict__ token_ids, int v_per_split, int splits,
                         StatQuad* __restrict__ partial, int group_m)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(lds_raw);
    int t_tile, split;
    if (!tile_coords((int)blockIdx.x, (Ntok + Cfg::BN - 1) / Cfg::BN, splits, group_m, t_tile, split)) return;
    const int t0 = t_tile * Cfg::BN;
    const int vb = split * v_per_split;
    const int ve = min(V, vb + v_per_split);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;

    float m[Cfg::NB], S[Cfg::NB], Sc[Cfg::NB], T[Cfg::NB], zy[Cfg::NB];
    int32_t y[Cfg::NB];
#pragma unroll
    for (int bj = 0; bj < Cfg::NB; ++bj) {
        m[bj] = kEmpty; S[bj] = 0.0f; Sc[bj] = 0.0f; T[bj] = 0.0f; zy[bj] = kEmpty;
        const int t = t0 + wn * Cfg::WN + bj * 32 + (lane & 31);
        y[bj] = t < Ntok ? token_ids[t] : -1;
    }

    for (int v0 = vb; v0 < ve; v0 += Cfg::BM) {
        f32x16 acc[Cfg::MB][Cfg::NB];
        gemm_tn_tile<Cfg>(Wt, Hd, V, v0, H, Hd, Ntok, t0, Hd, acc, lds);
        const int vrow0 = v0 + wm * Cfg::WM + 4 * (lane >> 5);
        // RAGGED: the tile reaches past the end of this workgroup's vocabulary range
        auto absorb_tile = [&](auto ragged_c) {
            constexpr bool RAGGED = decltype(ragged_c)::value;
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj) {
                float cm = kEmpty;
#pragma unroll
                for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int v = vrow0 + bi * 32 + 8 * (r >> 2) + (r & 3);
                        if (!RAGGED || v < ve) cm = fmaxf(cm, acc[bi][bj][r]);
                    }
                const float mn = fmaxf(m[bj], cm);
                const float d = m[bj] - mn;                   // <= 0
                const float sc = fast_exp2(d * kLog2e);
                float Tn = sc * fmaf(d, S[bj], T[bj]);
                const float Sn = sc * S[bj];
                const float Scn = sc * Sc[bj];
                float part = 0.0f;                            // this tile's terms first, then one TwoSum
#pragma unroll
                for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int v = vrow0 + bi * 32 + 8 * (r >> 2) + (r & 3);
                        const float x = acc[bi][bj][r] - mn;
                        const bool in = !RAGGED || v < ve;
                        const float e = in ? fast_exp2(x * kLog2e) : 0.0f;
                        part += e;
                        Tn = fmaf(e, in ? x : 0.0f, Tn);
                    }
                const float tsum = Sn + part;
                const float bv = tsum - Sn;
                const float err = (Sn - (tsum - bv)) + (part - bv);
                S[bj] = tsum; Sc[bj] = Scn + err; T[bj] = Tn; m[bj] = mn;
                // the chosen token's logit, if its row is one of this lane's in this tile (rare)
                const int dy = y[bj] - (v0 + wm * Cfg::WM);
                if (dy >= 0 && dy < Cfg::WM && ((dy >> 2) & 1) == (lane >> 5) && y[bj] < ve) {
#pragma unroll
                    for (int bi = 0; bi < Cfg::MB; ++bi)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (vrow0 + bi * 32 + 8 * (r >> 2) + (r & 3) == y[bj]) zy[bj] = acc[bi][bj][r];
                }
            }
        };
        if (v0 + Cfg::BM <= ve) absorb_tile(std::false_type{});
        else absorb_tile(std::true_type{});
    }

    // two lanes (lane, lane^32) share a token column; then the waves stacked along the vocabulary
    __shared__ float red[Cfg::WAVES_M][Cfg::BN][4];
#pragma unroll
    for (int bj = 0; bj < Cfg::NB; ++bj) {
        float mm = m[bj], SS = S[bj] + Sc[bj], TT = T[bj], zz = zy[bj];
        const float m2 = __shfl_xor(mm, 32), S2 = __shfl_xor(SS, 32), T2 = __shfl_xor(TT, 32), z2 = __shfl_xor(zz, 32);
        merge_nat(mm, SS, TT, m2, S2, T2);
        zz = fmaxf(zz, z2);
        if (lane < 32) {
            float* q = red[wm][wn * Cfg::WN + bj * 32 + lane];
            q[0] = mm; q[1] = SS; q[2] = TT; q[3] = zz;
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < Cfg::BN; c += Cfg::NT) {
        float mm = red[0][c][0], SS = red[0][c][1], TT = red[0][c][2], zz = red[0][c][3];
#pragma unroll
        for (int w = 1; w < Cfg::WAVES_M; ++w) {
            merge_nat(mm, SS, TT, red[w][c][0], red[w][c][1], red[w][c][2]);
            zz = fmaxf(zz, red[w][c][3]);
        }
        const int t = t0 + c;
        if (t < Ntok) partial[(int64_t)split * Ntok + t] = StatQuad{mm, SS, TT, zz};
    }
}

__global__ void lmhead_stats_merge_kernel(const StatQuad* __restrict__ partial, int splits, int Ntok, int V,
                                          const int32_t* __restrict__ token_ids, float* __restrict__ lse,
                                          float* __restrict__ logp, float* __restrict__ entropy)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= Ntok) return;
    StatQuad q = partial[t];
    for (int s = 1; s < splits; ++s) {
        const StatQuad p = partial[(int64_t)s * Ntok + t];
        merge_nat(q.m, q.S, q.T, p.m, p.S, p.T);
        q.zy = fmaxf(q.zy, p.zy);
    }
    const float lnS = logf(q.S);
    const int32_t y = token_ids[t];
    lse[t] = q.m + lnS;
    logp[t] = (y >= 0 && y < V) ? (q.zy - q.m) - lnS : __builtin_nanf("");
    entropy[t] = lnS - q.T / q.S;
}

// ---------------------------------------------------------------------------------------------
// backward: dz tiles of one vocabulary chunk, stored in both orientations
// ---------------------------------------------------------------------------------------------
// dz of one vocabulary chunk [vc0, vc0 + cw) (cw a multiple of 64; columns at or beyond V are
// written as zero): H [rows, Hd] holds the token rows of the product, Wt [V, Hd].  With a row map, H
// holds the gathered live rows and token column t stands for row row_map[t] of the per-token arrays.
struct DzArgs {
    const bf16_t* Wt; const bf16_t* H; int Hd; int V; int vc0; int cw;
    const int32_t* token_ids; const float* lse; const float* gcoef; float grad_out;
    bf16_t* dZc; int64_t ld_c;       // [token, v - vc0]
    bf16_t* dZcT; int64_t ld_t;      // [v - vc0, token]
    const int* row_map;
};

// The tile of workgroup `bid`.  Ntok: the number of token rows; t_tiles: token tiles to write (the
// last one is written in full, zeros beyond Ntok: the d_W product contracts over whole 64-column
// blocks of tokens).
template <class Cfg>
__device__ __forceinline__ void lmhead_dz_block(int bid, const DzArgs& a, int Ntok, int t_tiles, int group_m,
                                                unsigned char* lds_raw)
{
    const bf16_t* __restrict__ Wt = a.Wt;
    const bf16_t* __restrict__ H = a.H;
    const int Hd = a.Hd, V = a.V, vc0 = a.vc0, cw = a.cw;
    const int32_t* __restrict__ token_ids = a.token_ids;
    const float* __restrict__ lse = a.lse;
    const float* __restrict__ gcoef = a.gcoef;
    const float grad_out = a.grad_out;
    bf16_t* __restrict__ dZc = a.dZc;
    bf16_t* __restrict__ dZcT = a.dZcT;
    const int64_t ld_c = a.ld_c, ld_t = a.ld_t;
    const int* __restrict__ row_map = a.row_map;
    bf16_t* lds = reinterpret_cast<bf16_t*>(lds_raw);
    int v_tile, t_tile;
    if (!tile_coords(bid, (cw + Cfg::BM - 1) / Cfg::BM, t_tiles, group_m, v_tile, t_tile)) return;
    const int v0 = vc0 + v_tile * Cfg::BM;
    const int t0 = t_tile * Cfg::BN;
    const int vend = min(V, vc0 + cw);
    f32x16 acc[Cfg::MB][Cfg::NB];
    gemm_tn_tile<Cfg>(Wt, Hd, V, v0, H, Hd, Ntok, t0, Hd, acc, lds);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
    // Per token column of this lane:  dz = g (onehot - e^(z - lse)) = s (2^(z log2e + c) - |g| onehot)  with s = -sign(g),
    // c = log2|g| - lse log2e.  The magnitudes are computed and rounded; a negative s is applied to the packed pair by
    // flipping sign bits (rounding to nearest even is symmetric); a column without a gradient (zero coefficient, flagged row,
    // padding) is zeroed on the packed pair; the chosen token's term is patched in by the rare lanes whose rows hold it.
    // Per element that leaves one FMA, one exponential and half a conversion in the common path.
    const int v_wave = v0 + wm * Cfg::WM;
    const int t_wave = t0 + wn * Cfg::WN;
    float g_mag[Cfg::NB], c[Cfg::NB];
    uint32_t flip[Cfg::NB], keep[Cfg::NB];
    int dy[Cfg::NB];                              // row of the chosen token inside this wave's rows, -1 if not this lane's
#pragma unroll
    for (int bj = 0; bj < Cfg::NB; ++bj) {
        const int t = t_wave + bj * 32 + (lane & 31);
        g_mag[bj] = 0.0f; c[bj] = 0.0f; flip[bj] = 0u; keep[bj] = 0u; dy[bj] = -1;
        if (t < Ntok) {
            const int tt = row_map != nullptr ? row_map[t] : t;
            const float gg = gcoef[tt] * grad_out;
            const float l = lse[tt];
            const int32_t yy = token_ids[tt];
            if (row_has_gradient(gg, l, yy, V)) {
                const bool negate = gg > 0.0f;
                g_mag[bj] = negate ? -gg : gg;    // -|g|
                c[bj] = fmaf(-l, kLog2e, log2f(fabsf(gg)));
                flip[bj] = negate ? 0x80008000u : 0u;
                keep[bj] = 0xffffffffu;
                const int d = yy - v_wave;
                if (d >= 0 && d < Cfg::WM && ((d >> 2) & 1) == (lane >> 5) && yy < vend) dy[bj] = d;
            }
        }
    }
    const bool ragged = v0 + Cfg::BM > vend;      // uniform: the tile reaches past the end of the chunk

    // The tile leaves in both orientations, dZc[t, v] and dZc^T[v, t], as 16-byte row segments:
    // 64 vocabulary rows at a time go through the wave's share of LDS (the main loop's stages,
    // free by now), first laid out [v][t], then [t][v], and are read back row-wise.
    constexpr int NW = Cfg::NT / 64;
    constexpr int SA = Cfg::WN * 2 + 16;          // [v][t] row pitch in bytes (padded)
    constexpr int SB = 64 * 2 + 16;               // [t][v] row pitch
    constexpr int VPA = Cfg::WN * 2 / 16;         // 16-byte vectors per [v][t] row
    static_assert(Cfg::MB % 2 == 0, "64 vocabulary rows per round");
    static_assert((size_t)64 * SA <= Cfg::LDS_BYTES / NW && (size_t)Cfg::WN * SB <= Cfg::LDS_BYTES / NW, "round fits the wave's LDS share");
    unsigned char* slab = lds_raw + (size_t)wave * (Cfg::LDS_BYTES / NW);
#pragma unroll
    for (int h = 0; h < Cfg::MB / 2; ++h) {
        uint32_t pk[2][Cfg::NB][4][2];            // bf16 dz of this round: [block][column block][row quad] -> 4 rows
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float m[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) m[e] = fast_exp2(fmaf(acc[2 * h + b2][bj][4 * q + e], kLog2e, c[bj]));
                    if (ragged) {
                        const int v = v_wave + (2 * h + b2) * 32 + 8 * q + 4 * (lane >> 5);
#pragma unroll
                        for (int e = 0; e < 4; ++e) m[e] = (v + e < vend) ? m[e] : 0.0f;
                    }
                    pk[b2][bj][q][0] = (pack_bf16x2(m[0], m[1]) ^ flip[bj]) & keep[bj];
                    pk[b2][bj][q][1] = (pack_bf16x2(m[2], m[3]) ^ flip[bj]) & keep[bj];
                }
        // the chosen token's own term: only the lane whose rows of this round hold it
#pragma unroll
        for (int bj = 0; bj < Cfg::NB; ++bj) {
            if (dy[bj] >= h * 64 && dy[bj] < h * 64 + 64) {
#pragma unroll
                for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int row = (2 * h + b2) * 32 + 8 * q + 4 * (lane >> 5) + 2 * half;
                            if (dy[bj] == row || dy[bj] == row + 1) {
                                float m0 = fast_exp2(fmaf(acc[2 * h + b2][bj][4 * q + 2 * half], kLog2e, c[bj]));
                                float m1 = fast_exp2(fmaf(acc[2 * h + b2][bj][4 * q + 2 * half + 1], kLog2e, c[bj]));
                                if (dy[bj] == row) m0 += g_mag[bj]; else m1 += g_mag[bj];
                                pk[b2][bj][q][half] = pack_bf16x2(m0, m1) ^ flip[bj];
                            }
                        }
            }
        }
        // ---- [v][t]: rows of dZc^T
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = b2 * 32 + 8 * q + 4 * (lane >> 5);
                    unsigned char* p0 = slab + row * SA + (bj * 32 + (lane & 31)) * 2;
                    *reinterpret_cast<bf16_t*>(p0) = (bf16_t)(pk[b2][bj][q][0] & 0xffffu);
                    *reinterpret_cast<bf16_t*>(p0 + SA) = (bf16_t)(pk[b2][bj][q][0] >> 16);
                    *reinterpret_cast<bf16_t*>(p0 + 2 * SA) = (bf16_t)(pk[b2][bj][q][1] & 0xffffu);
                    *reinterpret_cast<bf16_t*>(p0 + 3 * SA) = (bf16_t)(pk[b2][bj][q][1] >> 16);
                }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 64 * VPA / 64; ++i) {
            const int row = (i * 64 + lane) / VPA, vec = (i * 64 + lane) % VPA;
            const u32x4 x = *reinterpret_cast<const u32x4*>(slab + row * SA + vec * 16);
            const int v = v_wave + h * 64 + row;
            const int t = t_wave + vec * 8;
            if (v < vc0 + cw && t < ld_t) *reinterpret_cast<u32x4*>(dZcT + (int64_t)(v - vc0) * ld_t + t) = x;
        }
        __syncthreads();
        // ---- [t][v]: rows of dZc
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
            for (int bj = 0; bj < Cfg::NB; ++bj)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = b2 * 32 + 8 * q + 4 * (lane >> 5);
                    const u32x2 two = {pk[b2][bj][q][0], pk[b2][bj][q][1]};
                    *reinterpret_cast<u32x2*>(slab + (bj * 32 + (lane & 31)) * SB + col * 2) = two;
                }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < Cfg::WN * 8 / 64; ++i) {
            const int row = (i * 64 + lane) / 8, vec = (i * 64 + lane) % 8;
            const u32x4 x = *reinterpret_cast<const u32x4*>(slab + row * SB + vec * 16);
            const int t = t_wave + row;
            const int v = v_wave + h * 64 + vec * 8;
            if (t < Ntok && v < vc0 + cw) *reinterpret_cast<u32x4*>(dZc + (int64_t)t * ld_c + (v - vc0)) = x;
        }
        __syncthreads();
    }
}

// One launch of the backward pass over the vocabulary chunks: the two products of the PREVIOUS
// chunk (d_W, then dHidden, from that chunk's dz buffers) and the dz tiles of the NEXT chunk
// (into the other pair of buffers) share the grid, longest tiles first.  Tile counts of the
// separate products rarely fill the 256 compute units a whole number of times (dHidden has only
// rows/256 x Hd/256 tiles); as parts of one launch the short dz tiles fill what the products leave
// idle.  Each part starts at a multiple of 8 workgroups, so a workgroup's XCD is its part-local
// id modulo 8.  n_live (device, may be NULL): the number of live rows, when rows were gathered.
struct BwdStepArgs {
    GemmArgs dw;       // C = d_W columns of the previous chunk: A = hidden^T [Hd, tokens], B = dz^T [cw, tokens]
    GemmArgs dh;       // C += dHidden accumulator: A = dz [tokens, cw], B = W rows restricted to the chunk [Hd, cw]
    DzArgs dz;
    int have_products, have_dz;
    int N;             // token rows (upper bound of the live count)
    int group_m;
    const int* n_live;
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WAVES_PER_SIMD, Cfg::WAVES_PER_SIMD)))
void lmhead_bwd_step_kernel(const BwdStepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    int rows = a.N;
    if (a.n_live != nullptr) rows = min(rows, *a.n_live);
    int bid = (int)blockIdx.x;
    if (a.have_products) {
        const int g_dw = (int)tile_grid((a.dw.M + Cfg::BM - 1) / Cfg::BM, (a.dw.N + Cfg::BN - 1) / Cfg::BN);
        if (bid < g_dw) {
            // contraction over the tokens: whole 64-column blocks up to the live count (zero terms beyond it)
            const int K = a.n_live != nullptr ? min(a.dw.K, (rows + 63) / 64 * 64) : a.dw.K;
            gemm_tn_block<Cfg, STORE_BF16>(bid, a.dw.A, a.dw.lda, a.dw.M, a.dw.B, a.dw.ldb, a.dw.N, K, a.dw.C, a.dw.ldc,
                                           a.dw.wide_rows, a.group_m, lds_raw);
            return;
        }
        bid -= g_dw;
        const int g_dh = rows > 0 ? (int)tile_grid((rows + Cfg::BM - 1) / Cfg::BM, (a.dh.N + Cfg::BN - 1) / Cfg::BN) : 0;
        if (bid < g_dh) {
            gemm_tn_block<Cfg, STORE_F32_ACCUM>(bid, a.dh.A, a.dh.lda, rows, a.dh.B, a.dh.ldb, a.dh.N, a.dh.K, a.dh.C, a.dh.ldc,
                                                a.dh.wide_rows, a.group_m, lds_raw);
            return;
        }
        bid -= g_dh;
    }
    if (a.have_dz && rows > 0) {
        const int t_tiles = a.n_live != nullptr ? (rows + Cfg::BN - 1) / Cfg::BN : (int)((a.dz.ld_t + Cfg::BN - 1) / Cfg::BN);
        lmhead_dz_block<Cfg>(bid, a.dz, rows, t_tiles, a.group_m, lds_raw);
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
// Tile shapes that are compiled in; ulorl_launch.gemm_tile selects one.
using TileLarge = GemmCfg<256, 256, 64, 2, 4, true>;   // eight waves (two per SIMD), wave tile 128 x 64, tiles copied global -> LDS directly
using TileSmall = GemmCfg<128, 128, 64, 2, 2>;         // four waves, wave tile 64 x 64, register-staged copies

#define ULORL_FOR_TILE(choice, ...)                              \
    switch (choice) {                                            \
    case 1: { using Cfg = TileSmall; __VA_ARGS__; } break;       \
    default: { using Cfg = TileLarge; __VA_ARGS__; } break;      \
    }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t round_up64(int64_t x) { return (x + 63) / 64 * 64; }

struct LmheadLayout {
    size_t wt, ht, dzc[2], dzct[2], dhacc, partial, token_ws, hc, pos, row_map, block_count, n_live, total;
    int64_t ldt;      // padded token count (leading dimension of Ht and dZc^T)
    int64_t ldc;      // padded chunk width (leading dimension of dZc)
    int splits;
    int v_per_split;
};

LmheadLayout lmhead_layout(int64_t N, int64_t Hd, int64_t V, int32_t R, int32_t chunk, int tile)
{
    int bm = 0, bn = 0;
    ULORL_FOR_TILE(tile, bm = Cfg::BM; bn = Cfg::BN)
    LmheadLayout L;
    L.ldt = round_up64(N);
    L.ldc = round_up64(chunk);
    const int64_t ttiles = (N + bn - 1) / bn;
    constexpr int kMaxSplits = 16;                          // the partial-statistics buffer holds this many slices
    int splits = (int)((1024 + ttiles - 1) / ttiles);       // aim at >= 1024 workgroups
    const int64_t vtiles = (V + bm - 1) / bm;
    if (splits > vtiles) splits = (int)vtiles;
    if (splits > kMaxSplits) splits = kMaxSplits;
    if (splits < 1) splits = 1;
    const int64_t tiles_per_split = (vtiles + splits - 1) / splits;
    L.v_per_split = (int)(tiles_per_split * bm);
    L.splits = (int)((vtiles + tiles_per_split - 1) / tiles_per_split);
    // sized for the largest split count any tile shape can ask for, so that the workspace
    // requirement does not depend on the launch options
    const size_t max_splits = kMaxSplits;
    size_t off = 0;
    L.wt = off;      off = align_up(off + (size_t)V * Hd * 2, 256);
    L.ht = off;      off = align_up(off + (size_t)Hd * L.ldt * 2, 256);
    // two pairs of dz buffers: one chunk's products read theirs while the next chunk's dz is written
    for (int b = 0; b < 2; ++b) {
        L.dzc[b] = off;  off = align_up(off + (size_t)N * L.ldc * 2, 256);
        L.dzct[b] = off; off = align_up(off + (size_t)L.ldc * L.ldt * 2, 256);
    }
    L.dhacc = off;   off = align_up(off + (size_t)N * Hd * 4, 256);
    L.partial = off; off = align_up(off + max_splits * (size_t)N * sizeof(StatQuad), 256);
    L.token_ws = off; off = align_up(off + workspace_layout(N, 0, R).total, 256);
    // backward over the live rows only: gathered hidden rows, row <-> position maps, scan scratch
    L.hc = off;          off = align_up(off + (size_t)N * Hd * 2, 256);
    L.pos = off;         off = align_up(off + (size_t)N * sizeof(int), 256);
    L.row_map = off;     off = align_up(off + (size_t)L.ldt * sizeof(int), 256);
    L.block_count = off; off = align_up(off + (size_t)((N + kLiveBlock - 1) / kLiveBlock) * sizeof(int), 256);
    L.n_live = off;      off = align_up(off + sizeof(int), 256);
    L.total = off;
    return L;
}

int32_t check_lmhead(const void* hidden, const void* W, int64_t N, int64_t Hd, int64_t V, int32_t chunk)
{
    if (!hidden || !W) return ULORL_ERR_NULL;
    // N and the chunk width become leading dimensions of GEMM operands (see kMaxLeadingDim)
    if (N <= 0 || N > kMaxLeadingDim - 256 || V <= 0 || V > 0x7fffffffLL || Hd <= 0 || Hd > (1 << 20)) return ULORL_ERR_SHAPE;
    if (Hd % 8 != 0 || V % 8 != 0) return ULORL_ERR_SHAPE;     // 16-byte rows of hidden, W and their transposes
    if (chunk <= 0 || chunk % 64 != 0 || chunk > kMaxLeadingDim - 256) return ULORL_ERR_SHAPE;
    if (((uintptr_t)hidden & 15u) != 0 || ((uintptr_t)W & 15u) != 0) return ULORL_ERR_ALIGN;
    return ULORL_OK;
}

// Raises the kernel's dynamic-LDS limit once per kernel and process (the runtime call is not a
// stream operation; keeping it out of later launches also keeps it out of stream captures that
// follow a warm-up call).
bool allow_lds_for(const void* kernel, size_t bytes)
{
    static std::mutex mu;
    static std::unordered_map<const void*, size_t> allowed;
    std::lock_guard<std::mutex> lock(mu);
    auto it = allowed.find(kernel);
    if (it != allowed.end() && it->second >= bytes) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
    allowed[kernel] = bytes;
    return true;
}

template <class Kernel>
bool allow_lds(Kernel k, size_t bytes)
{
    return allow_lds_for(reinterpret_cast<const void*>(k), bytes);
}

void launch_transpose(const bf16_t* src, int64_t ld_src, int rows, int cols, bf16_t* dst, int64_t ld_dst, int dst_cols,
                      hipStream_t st, const int* row_map = nullptr, const int* dyn_rows = nullptr)
{
    dim3 grid((unsigned)((dst_cols + 63) / 64), (unsigned)((cols + 63) / 64));
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, st, src, ld_src, rows, cols, dst, ld_dst, dst_cols,
                       row_map, dyn_rows);
}

template <int STORE>
GemmArgs gemm_args(const bf16_t* A, int64_t lda, int M, const bf16_t* B, int64_t ldb, int N, int K, void* C, int64_t ldc)
{
    const int eb = STORE == STORE_BF16 ? 2 : 4;
    GemmArgs g;
    g.A = A; g.lda = lda; g.M = M;
    g.B = B; g.ldb = ldb; g.N = N;
    g.K = K;
    g.C = C; g.ldc = ldc;
    g.wide_rows = (((uintptr_t)C & 15u) == 0 && (ldc * eb) % 16 == 0) ? 1 : 0;
    return g;
}

template <class Cfg, int STORE>
bool launch_gemm_cfg(const GemmArgs& g, int group_m, hipStream_t st)
{
    auto kern = gemm_tn_kernel<Cfg, STORE>;
    if (!allow_lds(kern, Cfg::LDS_BYTES)) return false;
    dim3 grid(tile_grid((g.M + Cfg::BM - 1) / Cfg::BM, (g.N + Cfg::BN - 1) / Cfg::BN));
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::NT), Cfg::LDS_BYTES, st, g, group_m);
    return true;
}

template <int STORE>
bool launch_gemm(const LaunchOpts& o, const bf16_t* A, int64_t lda, int M, const bf16_t* B, int64_t ldb, int N, int K,
                 void* C, int64_t ldc, hipStream_t st)
{
    const GemmArgs g = gemm_args<STORE>(A, lda, M, B, ldb, N, K, C, ldc);
    bool ok = false;
    ULORL_FOR_TILE(o.gemm_tile, ok = (launch_gemm_cfg<Cfg, STORE>(g, o.gemm_group_m, st)))
    return ok;
}

template <class Cfg>
bool launch_stats_cfg(const bf16_t* Wt, const bf16_t* H, int Hd, int V, int N, const int32_t* token_ids,
                      const LmheadLayout& L, StatQuad* partial, int group_m, hipStream_t st)
{
    auto kern = lmhead_stats_kernel<Cfg>;
    if (!allow_lds(kern, Cfg::LDS_BYTES)) return false;
    dim3 grid(tile_grid((N + Cfg::BN - 1) / Cfg::BN, L.splits));
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::NT), Cfg::LDS_BYTES, st, Wt, H, Hd, V, N, token_ids, L.v_per_split, L.splits,
                       partial, group_m);
    return true;
}

template <class Cfg>
bool launch_bwd_step_cfg(const BwdStepArgs& a, hipStream_t st)
{
    auto kern = lmhead_bwd_step_kernel<Cfg>;
    if (!allow_lds(kern, Cfg::LDS_BYTES)) return false;
    // the largest grid the live count allows; workgroups beyond the actual tiles return at once
    unsigned grid = 0;
    if (a.have_products) {
        grid += tile_grid((a.dw.M + Cfg::BM - 1) / Cfg::BM, (a.dw.N + Cfg::BN - 1) / Cfg::BN);
        grid += tile_grid((a.N + Cfg::BM - 1) / Cfg::BM, (a.dh.N + Cfg::BN - 1) / Cfg::BN);
    }
    if (a.have_dz) grid += tile_grid((a.dz.cw + Cfg::BM - 1) / Cfg::BM, (int)((a.dz.ld_t + Cfg::BN - 1) / Cfg::BN));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, st, a);
    return true;
}

}  // namespace

extern "C" {

int32_t ulorl_gemm_tn_bf16(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                           float* C, int64_t ldc, const ulorl_launch* launch, void* hip_stream)
{
    if (!A || !B || !C) return ULORL_ERR_NULL;
    LaunchOpts opts;
    const int32_t lrc = resolve_launch(launch, &opts);
    if (lrc != ULORL_OK) return lrc;
    if (M <= 0 || N <= 0 || K <= 0 || M > 0x7fffffffLL || N > 0x7fffffffLL || K > 0x7fffffffLL) return ULORL_ERR_SHAPE;
    if (K % 8 != 0 || lda % 8 != 0 || ldb % 8 != 0 || lda < K || ldb < K || ldc < N) return ULORL_ERR_SHAPE;
    if (lda > kMaxLeadingDim || ldb > kMaxLeadingDim) return ULORL_ERR_SHAPE;
    if (((uintptr_t)A & 15u) != 0 || ((uintptr_t)B & 15u) != 0) return ULORL_ERR_ALIGN;
    if (!launch_gemm<STORE_F32>(opts, (const bf16_t*)A, lda, (int)M, (const bf16_t*)B, ldb, (int)N, (int)K, C, ldc,
                                (hipStream_t)hip_stream))
        return ULORL_ERR_HIP;
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

size_t ulorl_lmhead_workspace_bytes(int64_t N, int64_t Hd, int64_t V, int32_t R, int32_t vocab_chunk)
{
    if (N <= 0 || N > 0x7fffffffLL || Hd <= 0 || V <= 0 || R <= 0 || vocab_chunk <= 0 || vocab_chunk % 64 != 0) return 0;
    return lmhead_layout(N, Hd, V, R, vocab_chunk, 0).total;      // the same for every tile shape
}

int32_t ulorl_lmhead_token_loss_fwd(const void* hidden, const void* W, int64_t N, int64_t Hd, int64_t V,
                                    int32_t vocab_chunk, const int32_t* token_ids, const int32_t* cu_seqlens,
                                    int32_t R, const int32_t* segment_ids, const float* old_logp,
                                    const float* advantages, const ulorl_params* p, float* loss, float* logp,
                                    float* entropy, float* lse, float* gcoef, uint8_t* mpt_mask, float* ratio,
                                    int32_t* segment_out, float* resp_entropy, uint8_t* resp_gate, int64_t* counters,
                                    const ulorl_segment_stats* seg_stats, void* workspace, size_t workspace_bytes,
                                    const ulorl_launch* launch, void* hip_stream)
{
    int32_t rc = check_lmhead(hidden, W, N, Hd, V, vocab_chunk);
    if (rc != ULORL_OK) return rc;
    if (!token_ids || !logp || !entropy || !lse) return ULORL_ERR_NULL;
    LaunchOpts opts;
    rc = resolve_launch(launch, &opts);
    if (rc != ULORL_OK) return rc;
    const bool stats_only = advantages == nullptr;      // lse, logp and entropy only (recording old log-probs)
    SegStatsArgs seg;
    seg.K = 0;
    if (!stats_only) {
        rc = check_objective_args(cu_seqlens, R, old_logp, p, loss, gcoef);
        if (rc != ULORL_OK) return rc;
        rc = resolve_segment_stats(seg_stats, N, &seg);
        if (rc != ULORL_OK) return rc;
    } else if (R <= 0) {
        R = 1;      // only sizes the workspace layout
    }
    const LmheadLayout L = lmhead_layout(N, Hd, V, R, vocab_chunk, opts.gemm_tile);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < L.total) return ULORL_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    bf16_t* Wt = (bf16_t*)(ws + L.wt);
    StatQuad* partial = (StatQuad*)(ws + L.partial);

    launch_transpose((const bf16_t*)W, V, (int)Hd, (int)V, Wt, Hd, (int)Hd, st);      // Wt[v, k] = W[k, v]
    bool ok = false;
    ULORL_FOR_TILE(opts.gemm_tile, ok = launch_stats_cfg<Cfg>(Wt, (const bf16_t*)hidden, (int)Hd, (int)V, (int)N, token_ids, L,
                                                              partial, opts.gemm_group_m, st))
    if (!ok) return ULORL_ERR_HIP;
    hipLaunchKernelGGL(lmhead_stats_merge_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, partial, L.splits,
                       (int)N, (int)V, token_ids, lse, logp, entropy);
    if (hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;
    if (stats_only) return ULORL_OK;

    const WorkspaceLayout wl = workspace_layout(N, 0, R);
    const TokenArgs a = make_token_args(N, V, token_ids, cu_seqlens, R, segment_ids, old_logp, advantages, p, logp,
                                        entropy, lse, gcoef, mpt_mask, ratio, segment_out, resp_entropy, resp_gate,
                                        ws + L.token_ws, wl, seg);
    launch_token_epilogue(a, wl, loss, counters, st);
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

int32_t ulorl_lmhead_token_loss_bwd(const void* hidden, const void* W, int64_t N, int64_t Hd, int64_t V,
                                    int32_t vocab_chunk, const int32_t* token_ids, const float* lse,
                                    const float* gcoef, float grad_out, void* d_hidden, void* d_W, void* workspace,
                                    size_t workspace_bytes, const ulorl_launch* launch, void* hip_stream)
{
    int32_t rc = check_lmhead(hidden, W, N, Hd, V, vocab_chunk);
    if (rc != ULORL_OK) return rc;
    LaunchOpts opts;
    rc = resolve_launch(launch, &opts);
    if (rc != ULORL_OK) return rc;
    if (!token_ids || !lse || !gcoef || !d_hidden || !d_W) return ULORL_ERR_NULL;
    if (((uintptr_t)d_hidden & 15u) != 0 || ((uintptr_t)d_W & 15u) != 0) return ULORL_ERR_ALIGN;
    const LmheadLayout L = lmhead_layout(N, Hd, V, 1, vocab_chunk, opts.gemm_tile);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < L.total) return ULORL_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    bf16_t* Wt = (bf16_t*)(ws + L.wt);
    bf16_t* Ht = (bf16_t*)(ws + L.ht);
    float* dHacc = (float*)(ws + L.dhacc);
    const bf16_t* H = (const bf16_t*)hidden;
    const bf16_t* Wp = (const bf16_t*)W;

    launch_transpose(Wp, V, (int)Hd, (int)V, Wt, Hd, (int)Hd, st);                    // Wt[v, k]
    const int64_t nh = N * Hd;
    hipLaunchKernelGGL(fill_zero_f32_kernel, dim3((unsigned)((nh / 4 + 255) / 256)), dim3(256), 0, st, dHacc, nh / 4);

    // Live rows (those with a non-zero coefficient): positions in order, gathered hidden rows and
    // their transpose.  ULORL_LAUNCH_DENSE_ROWS runs every row through the products instead.
    const bf16_t* Hrows = H;            // the token operand of the z product: [rows, Hd]
    const int* row_map = nullptr;
    const int* pos = nullptr;
    const int* n_live = nullptr;
    if (!opts.dense_rows) {
        int* posw = (int*)(ws + L.pos);
        int* mapw = (int*)(ws + L.row_map);
        int* cntw = (int*)(ws + L.block_count);
        int* nlw = (int*)(ws + L.n_live);
        bf16_t* Hc = (bf16_t*)(ws + L.hc);
        const int nblk = (int)((N + kLiveBlock - 1) / kLiveBlock);
        hipLaunchKernelGGL(live_count_kernel, dim3((unsigned)nblk), dim3(kLiveBlock), 0, st, gcoef, lse, token_ids, grad_out,
                           N, (int32_t)V, cntw);
        hipLaunchKernelGGL(live_scan_kernel, dim3(1), dim3(kLiveBlock), 0, st, cntw, nblk, nlw);
        hipLaunchKernelGGL(live_fill_kernel, dim3((unsigned)nblk), dim3(kLiveBlock), 0, st, gcoef, lse, token_ids, grad_out, N,
                           (int32_t)V, (const int*)cntw, posw, mapw);
        const int64_t nvec = N * (Hd / 8);
        hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st, H, (int)Hd,
                           (const int*)mapw, (const int*)nlw, N, Hc);
        launch_transpose(H, Hd, (int)N, (int)Hd, Ht, L.ldt, (int)L.ldt, st, mapw, nlw);   // Ht[k, j] = hidden[row_map[j], k], zero padded
        Hrows = Hc; row_map = mapw; pos = posw; n_live = nlw;
    } else {
        launch_transpose(H, Hd, (int)N, (int)Hd, Ht, L.ldt, (int)L.ldt, st);              // Ht[k, t], zero padded
    }
    if (hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;

    // Chunk pipeline: launch c holds the dz tiles of chunk c and the two products of chunk c - 1.
    const int64_t n_chunks = (V + vocab_chunk - 1) / vocab_chunk;
    for (int64_t c = 0; c <= n_chunks; ++c) {
        BwdStepArgs a;
        memset(&a, 0, sizeof(a));
        a.N = (int)N;
        a.group_m = opts.gemm_group_m;
        a.n_live = n_live;
        if (c >= 1) {
            const int64_t vp = (c - 1) * vocab_chunk;
            const int cwp = (int)((V - vp < vocab_chunk) ? (V - vp) : vocab_chunk);
            const bf16_t* dZc = (const bf16_t*)(ws + L.dzc[(c - 1) & 1]);
            const bf16_t* dZcT = (const bf16_t*)(ws + L.dzct[(c - 1) & 1]);
            a.have_products = 1;
            // dW[k, vp + v] = sum_j Ht[k, j] dZc^T[v, j]
            a.dw = gemm_args<STORE_BF16>(Ht, L.ldt, (int)Hd, dZcT, L.ldt, cwp, (int)L.ldt, (bf16_t*)d_W + vp, V);
            // dHidden[j, k] += sum_v dZc[j, v] W[k, vp + v]          (j: live position, or the row itself)
            a.dh = gemm_args<STORE_F32_ACCUM>(dZc, L.ldc, (int)N, Wp + vp, V, (int)Hd, cwp, dHacc, Hd);
        }
        if (c < n_chunks) {
            const int64_t vc0 = c * vocab_chunk;
            const int cw = (int)((V - vc0 < vocab_chunk) ? (V - vc0) : vocab_chunk);
            a.have_dz = 1;
            a.dz.Wt = Wt; a.dz.H = Hrows; a.dz.Hd = (int)Hd; a.dz.V = (int)V; a.dz.vc0 = (int)vc0;
            a.dz.cw = (int)round_up64(cw);               // dz of the padding columns is written as zero
            a.dz.token_ids = token_ids; a.dz.lse = lse; a.dz.gcoef = gcoef; a.dz.grad_out = grad_out;
            a.dz.dZc = (bf16_t*)(ws + L.dzc[c & 1]); a.dz.ld_c = L.ldc;
            a.dz.dZcT = (bf16_t*)(ws + L.dzct[c & 1]); a.dz.ld_t = L.ldt;
            a.dz.row_map = row_map;
        }
        bool ok = false;
        ULORL_FOR_TILE(opts.gemm_tile, ok = launch_bwd_step_cfg<Cfg>(a, st))
        if (!ok || hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;
    }
    hipLaunchKernelGGL(dhidden_finish_kernel, dim3((unsigned)((nh / 8 + 255) / 256)), dim3(256), 0, st, (const float*)dHacc, pos,
                       N, (int)Hd, (bf16_t*)d_hidden);
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

}  // extern "C"
