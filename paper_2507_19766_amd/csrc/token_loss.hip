// Fused UloRL token loss for gfx950 (MI355X): streaming kernels and their C entry points.
//
// The kernels behind the calls declared in ulorl.h:
//   row_stats_kernel      one workgroup per token row streams the V logits once with 16-byte
//                         loads and keeps a per-lane online (max, sum-exp, sum-exp*z) triple in
//                         registers; lanes are merged with wave shuffles, waves through LDS.
//                         -> lse, chosen-token log-prob (Eq. 6 numerator), entropy (Sec. 3.2.2).
//   piece_stats_kernel, piece_merge_kernel
//                         the same statistics from the pieces of cluster_row_kernel (below), used
//                         by the forward call whenever it has a workspace: both paths then carry
//                         the same bits.
//   response_entropy_kernel, token_terms_kernel, loss_finalize_kernel
//                         O(N) epilogue: per-response mean entropy and gate, SAIS/POIS ratio
//                         (Sec. 3.1.2), clipped term (Eq. 7), MPT mask (Eq. MPTS / I_msk), the
//                         token-mean loss and d loss / d logp.  Fixed-order fp64 sums.
//   dlogits_chunk_kernel  the backward call: recomputes the softmax from the saved lse and writes
//                         g_t * (onehot - p) with one 16-byte vector per thread; rows with
//                         g_t == 0 are write-only.  Safe in place: each vector is read and then
//                         written by the same thread.
//   cluster_row_kernel    the one-call entry point: a row is split into pieces, one workgroup per
//                         piece keeps its piece in registers, the pieces exchange their partial
//                         (max, sum, weighted sum) through memory and each writes its share of
//                         the gradient: every logit is read once and written once.
//   defer_compact_kernel, dlogits_rows_kernel
//                         the rows the one-call path leaves until the entropy gate is known (the
//                         members of the MPT set), collected into a list and finished from it.
//   repair_rows_kernel, repair_pieces_kernel
//                         finish what a workgroup of cluster_row_kernel left undone because its
//                         bounded wait expired; they return at once when nothing was left.
//   fused_row_kernel      the same call by one workgroup per row, forward and backward back to
//                         back (rows too long for the cooperative kernel, or on request).
//
// The HBM stream is the bound; the per-element VALU budget is what has to stay under it, so
// the inner loops are: unpack, one FMA (scaled argument), one v_exp_f32, and two accumulate
// ops in the forward; unpack, FMA, v_exp_f32 and a pack in the backward.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "ulorl.h"
#include "ulorl_internal.hpp"

using namespace ulorl_detail;

// Every fused multiply-add in this file is written out as fmaf(): the error-free transforms
// below (rescale by exactly 1 when the max is unchanged, TwoSum) are wrong if the compiler
// fuses a rounded product into a neighbouring add.
#pragma clang fp contract(off)

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kEmpty = -1.0e30f;  // "no element seen yet"; finite so that 0 * kEmpty == 0
static_assert(kSegBlock == kTokBlock, "the per-segment diagnostics ride on the O(N) epilogue's workgroups");
// Kernels with several workgroups per row lay the rows over grid dimensions y (up to
// kRowsPerGridY) and z (up to 65535).
constexpr int64_t kRowsPerGridY = 32768;
constexpr int64_t kMaxRows = kRowsPerGridY * 65535;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ u32x4 load_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store_stream(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// ---------------------------------------------------------------------------------------------
// storage traits: how a 16-byte vector maps to fp32 values
// ---------------------------------------------------------------------------------------------
struct StoreBF16 {
    using elem = uint16_t;
    static constexpr int kPerVec = 8;
    static __device__ __forceinline__ void unpack(u32x4 v, float* f)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[2 * k] = __uint_as_float(v[k] << 16);
            f[2 * k + 1] = __uint_as_float(v[k] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        f32x2 x = {lo, hi};
        bf16x2 b = __builtin_convertvector(x, bf16x2);  // round-to-nearest-even pair convert
        return __builtin_bit_cast(uint32_t, b);
    }
    static __device__ __forceinline__ u32x4 pack(const float* f)
    {
        u32x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = pack2(f[2 * k], f[2 * k + 1]);
        return v;
    }
    static __device__ __forceinline__ float load1(const elem* p) { return __uint_as_float(((uint32_t)*p) << 16); }
    static __device__ __forceinline__ void store1(elem* p, float x) { *p = (elem)(pack2(x, 0.0f) & 0xffffu); }
    // a vector of -9.95e29 (bf16 0xF149), used as padding that contributes nothing to a row's sums
    static __device__ __forceinline__ u32x4 filler() { return u32x4{0xf149f149u, 0xf149f149u, 0xf149f149u, 0xf149f149u}; }
    static __device__ __forceinline__ u32x4 sign_bits() { return u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u}; }
};

struct StoreF32 {
    using elem = float;
    static constexpr int kPerVec = 4;
    static __device__ __forceinline__ void unpack(u32x4 v, float* f)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) f[k] = __uint_as_float(v[k]);
    }
    static __device__ __forceinline__ u32x4 pack(const float* f)
    {
        u32x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __float_as_uint(f[k]);
        return v;
    }
    static __device__ __forceinline__ float load1(const elem* p) { return *p; }
    static __device__ __forceinline__ void store1(elem* p, float x) { *p = x; }
    static __device__ __forceinline__ u32x4 filler()
    {
        const uint32_t b = __float_as_uint(kEmpty);
        return u32x4{b, b, b, b};
    }
    static __device__ __forceinline__ u32x4 sign_bits() { return u32x4{0x80000000u, 0x80000000u, 0x80000000u, 0x80000000u}; }
};

// ---------------------------------------------------------------------------------------------
// online softmax statistics
// ---------------------------------------------------------------------------------------------
// Per lane: m = running max, mL = fl(m * log2e), S + Sc = sum 2^(z*log2e - mL),
// T = sum 2^(z*log2e - mL) * (z*log2e - mL)   (log2 units, <= 0).
//
// A peaked row has one term equal to 1 and ~V terms of 1e-8: added one by one to a running
// fp32 sum near 1 they would vanish below half an ulp.  So the terms of a chunk are first
// summed as a pairwise tree (the big term meets only log2(chunk) partial sums), and the chunk
// total is added to the running sum with an error-free TwoSum whose residual is carried in Sc.
struct LaneAcc {
    float m, mL, S, Sc, T;
};

template <int COUNT>
__device__ __forceinline__ void absorb(const float* f, LaneAcc& a)
{
    static_assert((COUNT & (COUNT - 1)) == 0, "chunk size must be a power of two");
    float cm = f[0];
#pragma unroll
    for (int k = 1; k < COUNT; ++k) cm = fmaxf(cm, f[k]);
    // rescale the running sums if this chunk raises the lane's max (branch-free; one exp per chunk)
    const float mn = fmaxf(a.m, cm);
    const float mLn = mn * kLog2e;
    const float d = a.mL - mLn;  // <= 0
    const float sc = fast_exp2(d);
    float T = sc * fmaf(d, a.S, a.T);
    const float S = sc * a.S;
    const float Sc = sc * a.Sc;
    float e[COUNT];
#pragma unroll
    for (int k = 0; k < COUNT; ++k) {
        const float x = fmaf(f[k], kLog2e, -mLn);
        e[k] = fast_exp2(x);
        T = fmaf(e[k], x, T);
    }
#pragma unroll
    for (int w = COUNT / 2; w >= 1; w >>= 1) {
#pragma unroll
        for (int k = 0; k < w; ++k) e[k] += e[k + w];
    }
    // TwoSum(S, e[0])
    const float t = S + e[0];
    const float bv = t - S;
    const float err = (S - (t - bv)) + (e[0] - bv);
    a.S = t;
    a.Sc = Sc + err;
    a.T = T;
    a.m = mn;
    a.mL = mLn;
}

// (m, S, T) with T in log2 units relative to m; exact when the two maxima coincide.
__device__ __forceinline__ void merge(float& m, float& S, float& T, float m2, float S2, float T2)
{
    const float M = fmaxf(m, m2);
    const float d1 = (m - M) * kLog2e;
    const float d2 = (m2 - M) * kLog2e;
    const float s1 = fast_exp2(d1);
    const float s2 = fast_exp2(d2);
    T = s1 * fmaf(d1, S, T) + s2 * fmaf(d2, S2, T2);
    S = s1 * S + s2 * S2;
    m = M;
}

// Row statistics of one row by one workgroup.  CACHED selects ordinary loads (the row stays in
// the L2 / memory-side cache for a second read by the same workgroup) instead of streaming
// non-temporal ones.  The result (max, sum, weighted sum in log2 units) is valid on thread 0.
struct RowStats {
    float m, S, T;
};

template <class Tr, int NT, int U, bool CACHED>
__device__ __forceinline__ RowStats row_stats_core(const typename Tr::elem* __restrict__ rowp, int32_t V)
{
    constexpr int E = Tr::kPerVec;
    constexpr int NW = NT / 64;
    const u32x4* vp = reinterpret_cast<const u32x4*>(rowp);
    const int nvec = V / E;
    const int tid = threadIdx.x;

    LaneAcc a = {kEmpty, kEmpty * kLog2e, 0.0f, 0.0f, 0.0f};

    int i = tid;
    for (; i + (U - 1) * NT < nvec; i += U * NT) {
        u32x4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) v[k] = CACHED ? vp[i + k * NT] : load_stream(vp + i + k * NT);
        float f[U * E];
#pragma unroll
        for (int k = 0; k < U; ++k) Tr::unpack(v[k], f + k * E);
        absorb<U * E>(f, a);
    }
    for (; i < nvec; i += NT) {
        float f[E];
        Tr::unpack(CACHED ? vp[i] : load_stream(vp + i), f);
        absorb<E>(f, a);
    }
    if (tid == NT - 1) {  // ragged tail when V is not a multiple of the vector width
        for (int j = nvec * E; j < V; ++j) {
            float f = Tr::load1(rowp + j);
            absorb<1>(&f, a);
        }
    }

    // The fused argument z*log2e - mL differs from (z - m)*log2e by the rounding residual of
    // mL, the same for every term of the lane: take it out once so that the term of the
    // maximum is exactly 1.
    const float delta = fmaf(a.m, kLog2e, -a.mL);
    const float un = fast_exp2(-delta);
    float m = a.m;
    float S = un * (a.S + a.Sc);
    float T = un * fmaf(-delta, a.S, a.T);

#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(m, off);
        const float S2 = __shfl_xor(S, off);
        const float T2 = __shfl_xor(T, off);
        merge(m, S, T, m2, S2, T2);
    }
    __shared__ float sm[NW], sS[NW], sT[NW];
    if ((tid & 63) == 0) {
        sm[tid >> 6] = m;
        sS[tid >> 6] = S;
        sT[tid >> 6] = T;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < NW; ++w) merge(m, S, T, sm[w], sS[w], sT[w]);
    }
    return RowStats{m, S, T};
}

// lse, chosen-token log-prob and entropy from the merged statistics (thread 0 only).
template <class Tr>
__device__ __forceinline__ void finish_row(const RowStats& st, const typename Tr::elem* rowp, int32_t V, int32_t y,
                                           float& lse, float& lp, float& ent)
{
    const float lnS = logf(st.S);
    lp = __builtin_nanf("");
    if (y >= 0 && y < V) lp = (Tr::load1(rowp + y) - st.m) - lnS;
    lse = st.m + lnS;
    ent = lnS - (st.T * kLn2) / st.S;
}

template <class Tr, int NT, int U>
__global__ __launch_bounds__(NT) void row_stats_kernel(const typename Tr::elem* __restrict__ logits,
                                                       int64_t row_stride, int32_t V,
                                                       const int32_t* __restrict__ token_ids,
                                                       float* __restrict__ lse_out,
                                                       float* __restrict__ logp_out,
                                                       float* __restrict__ ent_out)
{
    const int64_t row = blockIdx.x;
    const typename Tr::elem* rowp = logits + row * row_stride;
    const RowStats st = row_stats_core<Tr, NT, U, false>(rowp, V);
    if (threadIdx.x == 0) {
        float lse, lp, ent;
        finish_row<Tr>(st, rowp, V, token_ids[row], lse, lp, ent);
        lse_out[row] = lse;
        logp_out[row] = lp;
        ent_out[row] = ent;
    }
}

// ---------------------------------------------------------------------------------------------
// backward stream
// ---------------------------------------------------------------------------------------------
// One row of dlogits by one workgroup: zeros if !live, else g * (onehot(y) - exp(z - l)).
template <class Tr, int NT, int U>
__device__ __forceinline__ void dlogits_core(const typename Tr::elem* rowp, typename Tr::elem* outp, int32_t V,
                                             bool live, float g, float l, int32_t y)
{
    constexpr int E = Tr::kPerVec;
    const u32x4* vp = reinterpret_cast<const u32x4*>(rowp);
    u32x4* op = reinterpret_cast<u32x4*>(outp);
    const int nvec = V / E;
    const int tid = threadIdx.x;

    if (!live) {  // masked / clipped / zero-advantage / invalid row: write-only
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < nvec; i += NT) store_stream(op + i, zero);
        if (tid == NT - 1)
            for (int j = nvec * E; j < V; ++j) Tr::store1(outp + j, 0.0f);
        return;
    }

    // -g * exp(z - lse) = -sign(g) * 2^(z*log2e + c),  c = log2|g| - lse*log2e.  The magnitudes are
    // computed and rounded, the chosen column adds -sign(g) * g, and a negative sign is applied to
    // the packed result by flipping sign bits (rounding to nearest even is symmetric): the same
    // sequence as in cluster_row_kernel, so both give the same bits, signs of zeros included.
    const float c = fmaf(-l, kLog2e, log2f(fabsf(g)));
    const bool negate = g > 0.0f;
    const float sgn = negate ? -1.0f : 1.0f;
    const float g_mag = negate ? -g : g;
    const u32x4 flip = negate ? Tr::sign_bits() : u32x4{0u, 0u, 0u, 0u};
    const int yvec = y / E;

    // Software-pipelined: the loads of trip i+1 are issued before the stores of trip i (loads and
    // stores share one in-order outstanding-operation counter, so a load issued behind a store is
    // only known to have returned once that store has been acknowledged).  Measured effect on a
    // whole-row loop: none to speak of -- the write pattern of row-per-workgroup loops is what
    // limits them (see dlogits_chunk_kernel).
    auto emit = [&](const u32x4& v, int vec_index) {
        float f[E];
        Tr::unpack(v, f);
#pragma unroll
        for (int e = 0; e < E; ++e) f[e] = fast_exp2(fmaf(f[e], kLog2e, c));
        if (vec_index == yvec) {
#pragma unroll
            for (int e = 0; e < E; ++e) f[e] += (e == y - yvec * E) ? g_mag : 0.0f;
        }
        store_stream(op + vec_index, Tr::pack(f) ^ flip);
    };
    int i = tid;
    if (i + (U - 1) * NT < nvec) {
        u32x4 cur[U];
#pragma unroll
        for (int k = 0; k < U; ++k) cur[k] = load_stream(vp + i + k * NT);
        for (; i + (2 * U - 1) * NT < nvec; i += U * NT) {
            u32x4 nxt[U];
#pragma unroll
            for (int k = 0; k < U; ++k) nxt[k] = load_stream(vp + i + (U + k) * NT);
#pragma unroll
            for (int k = 0; k < U; ++k) emit(cur[k], i + k * NT);
#pragma unroll
            for (int k = 0; k < U; ++k) cur[k] = nxt[k];
        }
#pragma unroll
        for (int k = 0; k < U; ++k) emit(cur[k], i + k * NT);
        i += U * NT;
    }
    for (; i < nvec; i += NT) emit(load_stream(vp + i), i);
    if (tid == NT - 1) {
        for (int j = nvec * E; j < V; ++j) {
            float x = sgn * fast_exp2(fmaf(Tr::load1(rowp + j), kLog2e, c));
            if (j == y) x += g;
            Tr::store1(outp + j, x);
        }
    }
}

__device__ __forceinline__ bool row_is_live(float g, float l, int32_t y, int32_t V)
{
    return (g != 0.0f) && (fabsf(g) <= 3.0e38f) && (fabsf(l) <= 3.0e38f) && y >= 0 && y < V;
}

// The backward call, by one-shot workgroups: 256 threads, one 16-byte vector per thread, 4 KB of
// one row per workgroup, consecutive workgroups on consecutive addresses.  Measured on MI355X, a
// read-modify-write stream moves 6.5 TB/s this way against 5.1 TB/s when each workgroup loops
// over a whole row (the concurrent writes then spread over thousands of rows).
// grid = (chunks per row, rows mod kRowsPerGridY, rows / kRowsPerGridY).
// One 4 KB chunk (256 threads x one 16-byte vector) of one row of the gradient.
template <class Tr>
__device__ __forceinline__ void dlogits_chunk_body(const typename Tr::elem* logits, int64_t row_stride, int32_t V, int64_t row,
                                                   int chunk, bool last_chunk, const int32_t* __restrict__ token_ids,
                                                   const float* __restrict__ lse, const float* __restrict__ gcoef,
                                                   float grad_out, typename Tr::elem* dlogits)
{
    constexpr int E = Tr::kPerVec;
    const float g = gcoef[row] * grad_out;
    const float l = lse[row];
    const int32_t y = token_ids[row];
    const bool live = row_is_live(g, l, y, V);
    const typename Tr::elem* rowp = logits + row * row_stride;
    typename Tr::elem* outp = dlogits + row * row_stride;
    const int nvec = V / E;
    const int i = chunk * 256 + threadIdx.x;
    const float c = live ? fmaf(-l, kLog2e, log2f(fabsf(g))) : 0.0f;
    const bool negate = g > 0.0f;              // see dlogits_core
    const float sgn = negate ? -1.0f : 1.0f;
    const float g_mag = negate ? -g : g;
    if (i < nvec) {
        u32x4* op = reinterpret_cast<u32x4*>(outp) + i;
        if (!live) {
            const u32x4 zero = {0u, 0u, 0u, 0u};
            store_stream(op, zero);
        } else {
            float f[E];
            Tr::unpack(load_stream(reinterpret_cast<const u32x4*>(rowp) + i), f);
#pragma unroll
            for (int e = 0; e < E; ++e) f[e] = fast_exp2(fmaf(f[e], kLog2e, c));
            const int yvec = y / E;
            if (i == yvec) {
#pragma unroll
                for (int e = 0; e < E; ++e) f[e] += (e == y - yvec * E) ? g_mag : 0.0f;
            }
            u32x4 o = Tr::pack(f);
            if (negate) o ^= Tr::sign_bits();
            store_stream(op, o);
        }
    }
    if (last_chunk && threadIdx.x == 255) {   // ragged tail of the row
        for (int j = nvec * E; j < V; ++j) {
            float x = 0.0f;
            if (live) {
                x = sgn * fast_exp2(fmaf(Tr::load1(rowp + j), kLog2e, c));
                if (j == y) x += g;
            }
            Tr::store1(outp + j, x);
        }
    }
}

template <class Tr>
__global__ __launch_bounds__(256) void dlogits_chunk_kernel(const typename Tr::elem* logits, int64_t row_stride,
                                                            int32_t V, int64_t N,
                                                            const int32_t* __restrict__ token_ids,
                                                            const float* __restrict__ lse,
                                                            const float* __restrict__ gcoef, float grad_out,
                                                            typename Tr::elem* dlogits)
{
    const int64_t row = (int64_t)blockIdx.z * kRowsPerGridY + blockIdx.y;
    if (row >= N) return;
    dlogits_chunk_body<Tr>(logits, row_stride, V, row, (int)blockIdx.x, blockIdx.x == gridDim.x - 1, token_ids, lse, gcoef,
                           grad_out, dlogits);
}

// The same for a list of rows (the rows the one-call path deferred until the entropy gate was
// known): a fixed grid of (chunks per row) x kListRowSlots workgroups walks the list, so the launch
// costs what the listed rows cost, not a scan of all rows.
constexpr int kListRowSlots = 128;
template <class Tr>
__global__ __launch_bounds__(256) void dlogits_rows_kernel(const typename Tr::elem* logits, int64_t row_stride, int32_t V,
                                                           const uint32_t* __restrict__ rows,
                                                           const uint32_t* __restrict__ n_rows,
                                                           const int32_t* __restrict__ token_ids,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ gcoef, float grad_out,
                                                           typename Tr::elem* dlogits)
{
    const uint32_t n = *n_rows;
    for (uint32_t k = blockIdx.y; k < n; k += gridDim.y)
        dlogits_chunk_body<Tr>(logits, row_stride, V, (int64_t)rows[k], (int)blockIdx.x, blockIdx.x == gridDim.x - 1, token_ids,
                               lse, gcoef, grad_out, dlogits);
}

// Collects the rows flagged in `defer` into a list (order arbitrary: each row is processed exactly
// once whatever its position).  *count must be zero before the launch.
__global__ __launch_bounds__(256) void defer_compact_kernel(const uint8_t* __restrict__ defer, int64_t N,
                                                            uint32_t* __restrict__ rows, uint32_t* __restrict__ count)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool flagged = t < N && defer[t] != 0;
    const unsigned long long ballot = __ballot(flagged);
    if (ballot == 0ull) return;
    const int lane = threadIdx.x & 63;
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(count, (uint32_t)__popcll(ballot));
    base = __shfl(base, 0);
    if (flagged) rows[base + __popcll(ballot & ((1ull << lane) - 1ull))] = (uint32_t)t;
}

// ---------------------------------------------------------------------------------------------
// O(N) epilogue of the forward call
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ double shfl_xor_f64(double x, int off)
{
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return __hiloint2double(hi, lo);
}

// Everything about one token that does not depend on the entropy gate (Sec. 3.1.2 ratio,
// Eq. 7 clipped term, Eq. MPTS membership, coefficient assuming the token is not masked).
// Used by the O(N) epilogue and by the fused forward+backward kernel, so both take the same
// decisions bit for bit.
struct TokenEval {
    double r, s;    // importance ratio, clipped surrogate term
    float g;        // d loss / d logp if the token is kept
    bool positive;  // A > 0
    bool mpt;       // positive and p >= tau: member of the MPT set
    bool active;    // unclipped branch attains the min: gradient flows
};

__device__ __forceinline__ TokenEval token_eval(float lpf, float advf, float oldf, int is_mode, double eps_low,
                                                double eps_high, double log_tau, double inv_D)
{
    // Kept short: in the row-cooperative kernel one thread evaluates it while its workgroup waits.
    // p >= tau is tested as logp >= ln(tau); the ratio is one hardware exp2 (relative error ~2e-7).
    TokenEval ev;
    const double A = (double)advf;
    ev.positive = A > 0.0;
    ev.mpt = ev.positive && ((double)lpf >= log_tau);
    ev.r = (is_mode == ULORL_IS_POIS) ? 1.0 : (double)fast_exp2((lpf - oldf) * kLog2e);
    const double c = fmin(fmax(ev.r, 1.0 - eps_low), 1.0 + eps_high);
    const double u = ev.r * A, v = c * A;
    ev.active = u <= v;
    ev.s = ev.active ? u : v;
    ev.g = ev.active ? (float)(-(ev.r * A) * inv_D) : 0.0f;
    return ev;
}

__device__ __forceinline__ bool not_finite(float x) { return !(fabsf(x) <= 3.0e38f); }

// Fixed-shape tree: lanes by xor-shuffle, then waves through LDS in index order.
template <int NT>
__device__ __forceinline__ double block_sum_f64(double x, double* scratch)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += shfl_xor_f64(x, off);
    const int tid = threadIdx.x;
    __syncthreads();
    if ((tid & 63) == 0) scratch[tid >> 6] = x;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) s += scratch[w];
    return s;
}

template <int NT>
__device__ __forceinline__ long long block_sum_i64(long long x, long long* scratch)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int lo = (int)(x & 0xffffffffll), hi = (int)(x >> 32);
        lo = __shfl_xor(lo, off);
        hi = __shfl_xor(hi, off);
        x += ((long long)hi << 32) | (unsigned int)lo;
    }
    const int tid = threadIdx.x;
    __syncthreads();
    if ((tid & 63) == 0) scratch[tid >> 6] = x;
    __syncthreads();
    long long s = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) s += scratch[w];
    return s;
}

// Bitwise OR of the status bits over the workgroup (__syncthreads_or is a logical OR).
__device__ __forceinline__ int block_or_bits(int flags)
{
    int r = 0;
#pragma unroll
    for (int bit = 1; bit <= 8; bit <<= 1) r |= __syncthreads_or(flags & bit) ? bit : 0;
    return r;
}

__device__ __forceinline__ bool response_bounds_ok(const int32_t* cu, int i, int32_t R, int64_t N)
{
    const int64_t b = cu[i], e = cu[i + 1];
    return b >= 0 && e >= b && e <= N && (i != 0 || b == 0) && (i != R - 1 || e == N);
}

// Single workgroup: is cu_seqlens well formed?  (The fused kernel needs the answer before it
// writes any gradient.)
__global__ __launch_bounds__(kTokBlock) void cu_check_kernel(const int32_t* cu, int32_t R, int64_t N, uint32_t* badcu,
                                                             uint32_t* defer_count)
{
    if (threadIdx.x == 0) *defer_count = 0u;       // the list of deferred rows starts empty
    int bad = 0;
    for (int i = threadIdx.x; i < R; i += kTokBlock) bad |= response_bounds_ok(cu, i, R, N) ? 0 : 1;
    bad = __syncthreads_or(bad);
    if (threadIdx.x == 0) *badcu = bad ? 1u : 0u;
}

// One workgroup per response: sum of the token entropies (Sec. 3.2.2, H-bar_i numerator) and a
// sanity check of the response's bounds.
__global__ __launch_bounds__(kTokBlock) void response_entropy_kernel(TokenArgs a)
{
    __shared__ double scratch[kTokBlock / 64];
    const int i = blockIdx.x;
    const int64_t b = a.cu[i], e = a.cu[i + 1];
    const bool ok = response_bounds_ok(a.cu, i, a.R, a.N);
    double s = 0.0;
    if (ok)
        for (int64_t t = b + threadIdx.x; t < e; t += kTokBlock) s += (double)a.entropy[t];
    s = block_sum_f64<kTokBlock>(s, scratch);
    if (threadIdx.x == 0) {
        a.hsum[i] = s;
        a.rflags[i] = ok ? 0u : 1u;
    }
}

__global__ __launch_bounds__(kTokBlock) void token_terms_kernel(TokenArgs a)
{
    extern __shared__ double seg_table[];       // [K][7], only when the per-segment diagnostics are wanted
    __shared__ double scratch[kTokBlock / 64];
    __shared__ long long iscratch[kTokBlock / 64];
    const int tid = threadIdx.x;

    // call-wide facts every block derives identically: any malformed response, global entropy
    int badcu = 0;
    double hall = 0.0;
    for (int i = tid; i < a.R; i += kTokBlock) {
        badcu |= (int)a.rflags[i];
        hall += a.hsum[i];
    }
    badcu = __syncthreads_or(badcu);
    double hglobal = 0.0;
    if (a.gate_mode == ULORL_GATE_GLOBAL) hglobal = block_sum_f64<kTokBlock>(hall, scratch) / (double)a.N;

    const int64_t t = (int64_t)blockIdx.x * kTokBlock + tid;
    double contrib = 0.0;
    long long n_mask = 0, n_clip = 0, n_pos = 0, flags = badcu ? ULORL_STATUS_BAD_CU : 0;
    // what the per-segment diagnostics see of this token: exactly the values the call stores
    float g_out = 0.0f, r_out = 0.0f;
    uint8_t m_out = 0;
    int32_t sg_seg = 0;
    float sg_logp = 0.0f, sg_ent = 0.0f, sg_adv = 0.0f, sg_old = 0.0f;

    if (t < a.N) {
        // response of token t: largest i with cu[i] <= t
        int lo = 0, hi = a.R;  // invariant: cu[lo] <= t < cu[hi] for well-formed input
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((int64_t)a.cu[mid] <= t) lo = mid; else hi = mid;
        }
        const int i = lo;
        const int64_t b = a.cu[i];
        const int64_t L = (int64_t)a.cu[i + 1] - b;

        int gate;
        double hbar = 0.0;
        if (!badcu && L > 0) hbar = a.hsum[i] / (double)L;
        switch (a.gate_mode) {
        case ULORL_GATE_PER_RESPONSE: gate = (!badcu && L > 0) && (hbar < a.sigma); break;
        case ULORL_GATE_GLOBAL: gate = hglobal < a.sigma; break;
        case ULORL_GATE_ALWAYS: gate = 1; break;
        default: gate = 0; break;
        }
        const int32_t seg = a.segment_ids ? a.segment_ids[t]
                                          : (a.seg_len > 0 && !badcu ? (int32_t)((t - b) / a.seg_len) : 0);
        if (a.seg_out) a.seg_out[t] = seg;

        const float lpf = a.logp[t];
        const float hf = a.entropy[t];
        const float lf = a.lse[t];
        const int32_t y = a.token_ids[t];
        const bool bad_tok = (y < 0 || y >= a.V);
        const bool nonfinite = !(fabsf(lpf) <= 3.0e38f) || !(fabsf(hf) <= 3.0e38f) || !(fabsf(lf) <= 3.0e38f);
        if (bad_tok) flags |= ULORL_STATUS_BAD_TOKEN;
        if (!bad_tok && nonfinite) flags |= ULORL_STATUS_NONFINITE;

        sg_seg = seg; sg_logp = lpf; sg_ent = hf; sg_adv = a.adv[t];
        sg_old = (a.old_logp != nullptr) ? a.old_logp[t] : 0.0f;
        if (!bad_tok && !nonfinite && !badcu) {
            const TokenEval ev = token_eval(lpf, a.adv[t], a.is_mode == ULORL_IS_POIS ? 0.0f : a.old_logp[t],
                                            a.is_mode, a.eps_low, a.eps_high, a.log_tau, a.inv_D);
            const bool I = gate && ev.mpt;
            contrib = I ? 0.0 : ev.s;
            g_out = I ? 0.0f : ev.g;
            r_out = (float)ev.r;
            m_out = I ? 1 : 0;
            n_mask = I;
            n_clip = !ev.active;
            n_pos = ev.positive;
        }
        a.gcoef[t] = g_out;
        if (a.ratio) a.ratio[t] = r_out;
        if (a.mask) a.mask[t] = m_out;
    }

    const double bs = block_sum_f64<kTokBlock>(contrib, scratch);
    const long long c0 = block_sum_i64<kTokBlock>(n_mask, iscratch);
    const long long c1 = block_sum_i64<kTokBlock>(n_clip, iscratch);
    const long long c2 = block_sum_i64<kTokBlock>(n_pos, iscratch);
    const int fl = block_or_bits((int)flags);
    if (tid == 0) {
        a.part_sum[blockIdx.x] = bs;
        a.part_cnt[4 * (int64_t)blockIdx.x + 0] = c0;
        a.part_cnt[4 * (int64_t)blockIdx.x + 1] = c1;
        a.part_cnt[4 * (int64_t)blockIdx.x + 2] = c2;
        a.part_cnt[4 * (int64_t)blockIdx.x + 3] = fl;
    }
    if (a.seg.K > 0) {      // uniform over the grid
        int k;
        double v[kSegStats], oor;
        seg_token_values(t < a.N, sg_seg, a.seg.K, r_out, sg_logp, a.old_logp != nullptr, sg_old, sg_ent, m_out, sg_adv,
                         a.eps_low, a.eps_high, k, v, oor);
        const double o = seg_block_partials(k, v, oor, a.seg.K, seg_table,
                                            a.seg.part + (int64_t)blockIdx.x * a.seg.K * kSegStats);
        if (tid == 0) a.seg.part_oor[blockIdx.x] = o;
    }
}

__global__ __launch_bounds__(kTokBlock) void loss_finalize_kernel(TokenArgs a, int64_t nblk, float* loss,
                                                                 int64_t* counters)
{
    __shared__ double scratch[kTokBlock / 64];
    __shared__ long long iscratch[kTokBlock / 64];
    const double* part_sum = a.part_sum;
    const int64_t* part_cnt = a.part_cnt;
    const double D = a.D;

    // per-response outputs: mean entropy and gate (same call-wide reductions as token_terms_kernel)
    {
        int badcu = 0;
        double hall = 0.0;
        for (int i = threadIdx.x; i < a.R; i += kTokBlock) {
            badcu |= (int)a.rflags[i];
            hall += a.hsum[i];
        }
        badcu = __syncthreads_or(badcu);
        double hglobal = 0.0;
        if (a.gate_mode == ULORL_GATE_GLOBAL) hglobal = block_sum_f64<kTokBlock>(hall, scratch) / (double)a.N;
        for (int i = threadIdx.x; i < a.R; i += kTokBlock) {
            const int64_t L = badcu ? 0 : (int64_t)a.cu[i + 1] - (int64_t)a.cu[i];
            const double hbar = L > 0 ? a.hsum[i] / (double)L : 0.0;
            int gate;
            switch (a.gate_mode) {
            case ULORL_GATE_PER_RESPONSE: gate = L > 0 && hbar < a.sigma; break;
            case ULORL_GATE_GLOBAL: gate = hglobal < a.sigma; break;
            case ULORL_GATE_ALWAYS: gate = 1; break;
            default: gate = 0; break;
            }
            if (a.resp_entropy) a.resp_entropy[i] = (float)hbar;
            if (a.resp_gate) a.resp_gate[i] = badcu ? 0 : (uint8_t)gate;
        }
    }
    double s = 0.0;
    long long c0 = 0, c1 = 0, c2 = 0;
    int fl = 0;
    for (int64_t k = threadIdx.x; k < nblk; k += kTokBlock) {
        s += part_sum[k];
        c0 += part_cnt[4 * k + 0];
        c1 += part_cnt[4 * k + 1];
        c2 += part_cnt[4 * k + 2];
        fl |= (int)part_cnt[4 * k + 3];
    }
    s = block_sum_f64<kTokBlock>(s, scratch);
    c0 = block_sum_i64<kTokBlock>(c0, iscratch);
    c1 = block_sum_i64<kTokBlock>(c1, iscratch);
    c2 = block_sum_i64<kTokBlock>(c2, iscratch);
    fl = block_or_bits(fl);
    if (threadIdx.x == 0) {
        if (a.sync_fail != nullptr && *a.sync_fail != 0u) fl |= ULORL_STATUS_SYNC;
        *loss = (float)(-s / D);
        if (counters) {
            counters[0] = c0;
            counters[1] = c1;
            counters[2] = c2;
            counters[3] = fl;
        }
    }
    if (a.seg.K > 0) {
        __shared__ double seg_scratch[kTokBlock];
        seg_finalize(a.seg, nblk, seg_scratch);
    }
}

// ---------------------------------------------------------------------------------------------
// fused forward + backward, one looping workgroup per row (the older kernel of the one-call path,
// selected with ULORL_TUNE_FUSED_CLUSTER = 0 and used for rows too long for the cooperative one)
// ---------------------------------------------------------------------------------------------
// One workgroup per row does both passes back to back: statistics with ordinary (cacheable)
// loads, then the gradient with the row read a second time while it is still in the L2 /
// memory-side cache, so HBM sees one read and one write per row.  This is possible whenever the
// row's coefficient does not depend on other rows: always for the ALWAYS / NEVER gates, and for
// every token outside the MPT set under the entropy gates.  MPT members under an entropy gate
// are left untouched and flagged in `defer`; dlogits_kernel finishes them once the gate is known.
struct FusedArgs {
    const int32_t* token_ids;
    const float* old_logp;
    const float* adv;
    float* lse;
    float* logp;
    float* entropy;
    uint8_t* defer;
    float* zy_row;          // [N] chosen logit of each row, kept for the repair pass (row-cooperative kernel only)
    const uint32_t* badcu;  // one word: non-zero if cu_seqlens is malformed (then nothing is trained)
    int32_t is_mode, gate_mode;
    double eps_low, eps_high, log_tau, inv_D;
    float grad_out;
};

// What the one-call path does with a row once its statistics are known: mode 0 = write zeros,
// 1 = write the gradient with coefficient g, 2 = leave the row to the filtered backward launch that
// follows the gate (a member of the MPT set under an entropy gate).
__device__ __forceinline__ int row_decision(const FusedArgs& a, int32_t y, int32_t V, float lse, float lp, float ent,
                                            float adv, float old, uint32_t badcu, float& g)
{
    g = 0.0f;
    const bool bad = (y < 0 || y >= V) || not_finite(lp) || not_finite(ent) || not_finite(lse) || badcu != 0;
    if (bad) return 0;
    const TokenEval ev = token_eval(lp, adv, old, a.is_mode, a.eps_low, a.eps_high, a.log_tau, a.inv_D);
    const bool gate_known = a.gate_mode == ULORL_GATE_ALWAYS || a.gate_mode == ULORL_GATE_NEVER;
    if (ev.mpt && !gate_known) return 2;
    const bool I = ev.mpt && a.gate_mode == ULORL_GATE_ALWAYS;
    g = (I ? 0.0f : ev.g) * a.grad_out;
    return row_is_live(g, lse, y, V) ? 1 : 0;
}

template <class Tr, int NT, int U>
__global__ __launch_bounds__(NT) void fused_row_kernel(const typename Tr::elem* logits, int64_t row_stride, int32_t V,
                                                       typename Tr::elem* dlogits, FusedArgs a)
{
    __shared__ float bc_g, bc_l;
    __shared__ int bc_mode;  // 0: write zeros, 1: write gradient, 2: deferred
    const int64_t row = blockIdx.x;
    const typename Tr::elem* rowp = logits + row * row_stride;
    const int32_t y = a.token_ids[row];
    const RowStats st = row_stats_core<Tr, NT, U, true>(rowp, V);
    if (threadIdx.x == 0) {
        float lse, lp, ent;
        finish_row<Tr>(st, rowp, V, y, lse, lp, ent);
        a.lse[row] = lse;
        a.logp[row] = lp;
        a.entropy[row] = ent;
        float g;
        const int mode = row_decision(a, y, V, lse, lp, ent, a.adv[row], a.is_mode == ULORL_IS_POIS ? 0.0f : a.old_logp[row],
                                      *a.badcu, g);
        a.defer[row] = mode == 2 ? 1 : 0;
        bc_g = g;
        bc_l = lse;
        bc_mode = mode;
    }
    __syncthreads();
    const int mode = bc_mode;
    if (mode == 2) return;
    dlogits_core<Tr, NT, U>(rowp, dlogits + row * row_stride, V, mode == 1, bc_g, bc_l, y);
}

// ---------------------------------------------------------------------------------------------
// fused forward + backward, one read and one write of HBM per row: row-cooperative workgroups
// ---------------------------------------------------------------------------------------------
// C workgroups of 256 threads share a row; each keeps its piece (VPT 16-byte vectors per thread)
// in registers, computes the piece's statistics, publishes them, waits for the other pieces',
// and turns its registers into the gradient.  Nothing is read twice, and because consecutive
// workgroups work on consecutive pieces of consecutive rows the chip reads and writes a narrow
// moving window of addresses (measured: 12.3 ms for 131072 x 151936 bf16, the rate of a plain
// one-shot copy; one workgroup per row reaches 16.3 ms).
//
// Exchange: piece c of a row owns two 64-bit words, {m, S} and {T, 1}, zero before the launch.
// Each is written and read with relaxed agent-scope atomics, and each carries its own validity
// (S >= 1 for a non-empty piece; the tag), so no ordering between memory locations and no cache
// maintenance is needed.  Workgroups are dispatched in order of their linear id and a row's
// pieces have consecutive ids, so the partners of a resident workgroup are resident or next in
// line; the wait is nevertheless bounded (spin_limit polls, seconds by default).  A workgroup whose
// wait expires writes NOTHING (in place, its piece of the logits stays intact), re-publishes its
// second word with the tag kTagPending and raises the sync_fail word; after the kernel every piece's
// statistics are in the slots, and the repair kernels below finish the row from them.  Every
// workgroup of a row that completes its wait merges the same pieces in the same order and therefore
// takes the same decisions; the repair pass merges them in that order too.
constexpr int kClusterThreads = 256;
constexpr int kClusterMaxPieces = 64;         // one polled piece per lane of a wave

// Absorbs vectors v[K .. VPT) in power-of-two groups, largest first (absorb<> wants a power of two).
template <class Tr, int VPT, int K>
__device__ __forceinline__ void absorb_vectors(const u32x4 (&v)[VPT], LaneAcc& acc)
{
    constexpr int REM = VPT - K;
    if constexpr (REM > 0) {
        constexpr int G = REM >= 8 ? 8 : REM >= 4 ? 4 : REM >= 2 ? 2 : 1;
        constexpr int E = Tr::kPerVec;
        float f[G * E];
#pragma unroll
        for (int q = 0; q < G; ++q) Tr::unpack(v[K + q], f + q * E);
        absorb<G * E>(f, acc);
        absorb_vectors<Tr, VPT, K + G>(v, acc);
    }
}

// Phase 1 of a piece: its vectors into registers (v) and its (max, sum, weighted sum), merged over
// the workgroup; the result is valid on thread 0 after the barrier this function ends with.
template <class Tr, int VPT>
__device__ __forceinline__ void piece_statistics(const u32x4* vp, const typename Tr::elem* rowp, int nvec, int32_t V,
                                                 int first, bool full, bool owns_tail, u32x4 (&v)[VPT],
                                                 float* sm, float* sS, float* sT, float& m, float& S, float& T)
{
    constexpr int NT = kClusterThreads;
    constexpr int E = Tr::kPerVec;
    const int tid = threadIdx.x;
    LaneAcc acc = {kEmpty, kEmpty * kLog2e, 0.0f, 0.0f, 0.0f};
    if (full) {
        const char* const piece_in = reinterpret_cast<const char*>(vp + first);
#pragma unroll
        for (int k = 0; k < VPT; ++k)
            v[k] = load_stream(reinterpret_cast<const u32x4*>(piece_in + (size_t)k * NT * 16 + (uint32_t)tid * 16u));
        absorb_vectors<Tr, VPT, 0>(v, acc);
    } else if (nvec - first >= NT) {
        // A row's last piece: every thread holds at least one vector.  Missing vectors are
        // replaced by a very negative finite filler, whose terms are exactly zero once the lane's
        // maximum is a real logit (guaranteed: the thread's first vector is real), so the piece
        // takes the same grouped arithmetic as a full one.
        const u32x4 filler = Tr::filler();
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int i = first + k * NT + tid;
            v[k] = filler;
            if (i < nvec) v[k] = load_stream(vp + i);
        }
        absorb_vectors<Tr, VPT, 0>(v, acc);
    } else {
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int i = first + k * NT + tid;
            if (i < nvec) {
                v[k] = load_stream(vp + i);
                float f[E];
                Tr::unpack(v[k], f);
                absorb<E>(f, acc);
            }
        }
    }
    if (owns_tail) {
        for (int j = nvec * E; j < V; ++j) {
            float f = Tr::load1(rowp + j);
            absorb<1>(&f, acc);
        }
    }
    const float delta = fmaf(acc.m, kLog2e, -acc.mL);
    const float un = fast_exp2(-delta);
    m = acc.m;
    S = un * (acc.S + acc.Sc);
    T = un * fmaf(-delta, acc.S, acc.T);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(m, off);
        const float S2 = __shfl_xor(S, off);
        const float T2 = __shfl_xor(T, off);
        merge(m, S, T, m2, S2, T2);
    }
    if ((tid & 63) == 0) {
        sm[tid >> 6] = m;
        sS[tid >> 6] = S;
        sT[tid >> 6] = T;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) merge(m, S, T, sm[w], sS[w], sT[w]);
    }
}

// The two words a piece publishes: {m, S} and {T, tag 1}.
__device__ __forceinline__ unsigned long long piece_word0(float m, float S)
{
    return ((unsigned long long)__float_as_uint(S) << 32) | __float_as_uint(m);
}
constexpr unsigned long long kTagPublished = 1, kTagPending = 3;   // pending = published, and the piece's gradient is not written yet
__device__ __forceinline__ unsigned long long piece_word1(float T, unsigned long long tag = kTagPublished)
{
    return (tag << 32) | __float_as_uint(T);
}

// Merge of a row's pieces by one wave: lane c < C brings piece c, the other lanes nothing; a fixed
// xor-shuffle tree, so every wave that merges the same pieces gets the same bits.
__device__ __forceinline__ void merge_pieces_tree(float& pm, float& pS, float& pT)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(pm, off);
        const float S2 = __shfl_xor(pS, off);
        const float T2 = __shfl_xor(pT, off);
        merge(pm, pS, pT, m2, S2, T2);
    }
}

// lse, chosen-token log-prob and entropy of a row from its merged pieces (T in log2 units).
__device__ __forceinline__ void finish_pieces(float pm, float pS, float pT, bool has_y, float zy, float& lse, float& lp,
                                              float& ent)
{
    const float lnS = logf(pS);
    lp = __builtin_nanf("");
    if (has_y) lp = (zy - pm) - lnS;
    lse = pm + lnS;
    ent = lnS - (pT * kLn2) / pS;
}

struct ClusterArgs {
    FusedArgs f;
    unsigned long long* slots;   // [N * C * 2]
    uint32_t* sync_fail;         // one word, set if any wait expired
    int64_t N;
    int32_t C;
    int32_t spin_limit;          // polls (~0.25 us each) before a wait is given up
};

template <class Tr, int VPT>
__global__ __launch_bounds__(kClusterThreads) void cluster_row_kernel(const typename Tr::elem* logits, int64_t row_stride,
                                                                      int32_t V, typename Tr::elem* dlogits,
                                                                      ClusterArgs a)
{
    constexpr int NT = kClusterThreads;
    constexpr int E = Tr::kPerVec;
    constexpr int P = NT * VPT;                 // vectors per piece
    const int c = blockIdx.x;
    const int C = a.C;
    const int64_t row = (int64_t)blockIdx.z * kRowsPerGridY + blockIdx.y;
    if (row >= a.N) return;
    const int tid = threadIdx.x;
    const typename Tr::elem* rowp = logits + row * row_stride;
    typename Tr::elem* outp = dlogits + row * row_stride;
    const u32x4* vp = reinterpret_cast<const u32x4*>(rowp);
    u32x4* op = reinterpret_cast<u32x4*>(outp);
    const int nvec = V / E;
    const int first = c * P;
    const bool full = first + P <= nvec;        // every thread holds VPT vectors
    const bool owns_tail = (c == C - 1) && (tid == NT - 1) && (nvec * E < V);

    // Per-row scalars, fetched first so that their latency hides under the row's loads.  The
    // chosen logit in particular must have arrived before this piece is published: from then
    // on a partner may overwrite the row (in place).
    const int32_t y = a.f.token_ids[row];
    const float adv_row = a.f.adv[row];
    const float old_row = a.f.is_mode == ULORL_IS_POIS ? 0.0f : a.f.old_logp[row];
    const uint32_t badcu = *a.f.badcu;
    float zy = 0.0f;
    if (tid == 0 && y >= 0 && y < V) zy = Tr::load1(rowp + y);
    if (tid == 0 && c == 0) a.f.zy_row[row] = zy;     // the repair pass cannot read it from a row overwritten in place

    // ---- phase 1: the piece into registers, its statistics (valid on thread 0)
    u32x4 v[VPT];
    __shared__ float sm[NT / 64], sS[NT / 64], sT[NT / 64];
    __shared__ float bc_g, bc_l;
    __shared__ int bc_mode;      // 0: write zeros, 1: write gradient, 2: deferred (leave the row alone)
    float m, S, T;
    piece_statistics<Tr, VPT>(vp, rowp, nvec, V, first, full, owns_tail, v, sm, sS, sT, m, S, T);

    // ---- exchange (first wave)
    if (tid < 64) {
        unsigned long long* slot = a.slots + (row * C) * 2;
        if (tid == 0) {
            __builtin_amdgcn_s_waitcnt(0);      // every load of this thread, the chosen logit included, has returned
            __hip_atomic_store(slot + 2 * c, piece_word0(m, S), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(slot + 2 * c + 1, piece_word1(T), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        float pm = kEmpty, pS = 0.0f, pT = 0.0f;
        int expired = 0;
        if (tid < C) {
            unsigned long long w0 = 0, w1 = 0;
            int spins = 0;
            for (;;) {
                if (w0 == 0) w0 = __hip_atomic_load(slot + 2 * tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (w1 == 0) w1 = __hip_atomic_load(slot + 2 * tid + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (w0 != 0 && w1 != 0) break;
                if (++spins >= a.spin_limit) { expired = 1; break; }
                __builtin_amdgcn_s_sleep(4);
            }
            if (!expired) {
                pm = __uint_as_float((uint32_t)w0);
                pS = __uint_as_float((uint32_t)(w0 >> 32));
                pT = __uint_as_float((uint32_t)w1);
            }
        }
        expired = __any(expired);
        merge_pieces_tree(pm, pS, pT);
        if (tid == 0) {
            if (expired) {
                // leave everything to the repair pass: nothing of this piece is written
                __hip_atomic_store(slot + 2 * c + 1, piece_word1(T, kTagPending), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *a.sync_fail = 1u;
                bc_mode = 2;
            } else {
                float lse, lp, ent, g;
                finish_pieces(pm, pS, pT, y >= 0 && y < V, zy, lse, lp, ent);
                const int mode = row_decision(a.f, y, V, lse, lp, ent, adv_row, old_row, badcu, g);
                if (c == 0) {
                    a.f.lse[row] = lse;
                    a.f.logp[row] = lp;
                    a.f.entropy[row] = ent;
                    a.f.defer[row] = mode == 2 ? 1 : 0;
                }
                bc_g = g;
                bc_l = lse;
                bc_mode = mode;
            }
        }
    }
    __syncthreads();

    // ---- phase 2: the gradient from the registers
    const int mode = bc_mode;
    if (mode == 2) return;
    if (mode == 0) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int i = first + k * NT + tid;
            if (i < nvec) store_stream(op + i, zero);
        }
        if (owns_tail)
            for (int j = nvec * E; j < V; ++j) Tr::store1(outp + j, 0.0f);
        return;
    }
    // dz = -g e^(z - lse) = s 2^(z log2e + cexp) with s = -sign(g), cexp = log2|g| - lse log2e.  The
    // magnitudes are computed and rounded; a negative s is applied to the packed result by flipping
    // sign bits (rounding to nearest even is symmetric), and the chosen column adds s*g before
    // that.  Specialised for (full piece, sign) so that the common case carries no guards, no sign
    // multiply and no per-vector address arithmetic (uniform base + lane offset).
    const float g = bc_g;
    const float cexp = fmaf(-bc_l, kLog2e, log2f(fabsf(g)));
    const bool negate = g > 0.0f;
    const float g_mag = negate ? -g : g;       // s * g
    const int ky = y / E - first - tid;        // this thread holds the chosen column in vector k iff ky == k * NT
    const int ey = y - (y / E) * E;
    char* const piece_out = reinterpret_cast<char*>(op + first);
    const uint32_t lane_off = (uint32_t)tid * 16u;
    auto emit_all = [&](auto full_c, auto neg_c) {
        constexpr bool FULL = decltype(full_c)::value;
        constexpr bool NEG = decltype(neg_c)::value;
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            if (FULL || first + k * NT + tid < nvec) {
                float f[E];
                Tr::unpack(v[k], f);
#pragma unroll
                for (int e = 0; e < E; ++e) f[e] = fast_exp2(fmaf(f[e], kLog2e, cexp));
                if (ky == k * NT) {
#pragma unroll
                    for (int e = 0; e < E; ++e) f[e] += (e == ey) ? g_mag : 0.0f;
                }
                u32x4 o = Tr::pack(f);
                if (NEG) o ^= Tr::sign_bits();
                store_stream(reinterpret_cast<u32x4*>(piece_out + (size_t)k * NT * 16 + lane_off), o);
            }
        }
    };
    if (full) {
        if (negate) emit_all(std::true_type{}, std::true_type{});
        else emit_all(std::true_type{}, std::false_type{});
    } else {
        if (negate) emit_all(std::false_type{}, std::true_type{});
        else emit_all(std::false_type{}, std::false_type{});
    }
    if (owns_tail) {
        // the tail's logits have not been overwritten: only this thread writes them
        const float sgn = negate ? -1.0f : 1.0f;
        for (int j = nvec * E; j < V; ++j) {
            float x = sgn * fast_exp2(fmaf(Tr::load1(rowp + j), kLog2e, cexp));
            if (j == y) x += g;
            Tr::store1(outp + j, x);
        }
    }
}

__global__ void fill_zero_u64_kernel(unsigned long long* p, int64_t n, uint32_t* flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
    if (i == 0) *flag = 0u;
}

// ---------------------------------------------------------------------------------------------
// repair pass of the row-cooperative kernel
// ---------------------------------------------------------------------------------------------
// Both kernels have a small fixed grid and return at once unless a wait expired (sync_fail).  By
// the time they run every piece of every row has published its statistics (a workgroup publishes
// before it waits), so a row's statistics can be formed exactly as a workgroup would have formed
// them; a pending piece's logits are intact because only its own workgroup writes them.
constexpr int kRepairRowGrid = 256;      // workgroups of 4 waves, one wave per row at a time
constexpr int kRepairPieceGrid = 2048;   // workgroups of kClusterThreads, one piece at a time

// Rows with a pending piece: their statistics, per-row outputs and deferral flag, as piece 0 would
// have written them (rewritten with the same bits if it did).
__global__ __launch_bounds__(256) void repair_rows_kernel(ClusterArgs a, int32_t V)
{
    if (*a.sync_fail == 0u) return;
    const int lane = threadIdx.x & 63;
    const int C = a.C;
    const uint32_t badcu = *a.f.badcu;
    for (int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); row < a.N; row += (int64_t)gridDim.x * 4) {
        float pm = kEmpty, pS = 0.0f, pT = 0.0f;
        int pending = 0;
        if (lane < C) {
            const unsigned long long w0 = a.slots[(row * C + lane) * 2], w1 = a.slots[(row * C + lane) * 2 + 1];
            pm = __uint_as_float((uint32_t)w0);
            pS = __uint_as_float((uint32_t)(w0 >> 32));
            pT = __uint_as_float((uint32_t)w1);
            pending = (w1 >> 32) == kTagPending;
        }
        if (!__any(pending)) continue;
        merge_pieces_tree(pm, pS, pT);
        if (lane == 0) {
            const int32_t y = a.f.token_ids[row];
            float lse, lp, ent, g;
            finish_pieces(pm, pS, pT, y >= 0 && y < V, a.f.zy_row[row], lse, lp, ent);
            const int mode = row_decision(a.f, y, V, lse, lp, ent, a.f.adv[row],
                                          a.f.is_mode == ULORL_IS_POIS ? 0.0f : a.f.old_logp[row], badcu, g);
            a.f.lse[row] = lse;
            a.f.logp[row] = lp;
            a.f.entropy[row] = ent;
            a.f.defer[row] = mode == 2 ? 1 : 0;
        }
    }
}

// Pending pieces of rows that were not deferred as a whole: their share of the gradient, with the
// arithmetic of the backward call (the same bits the piece's own workgroup would have written).
// Runs after the O(N) epilogue (gcoef) and after the filtered backward launch of the deferred rows.
template <class Tr>
__global__ __launch_bounds__(kClusterThreads) void repair_pieces_kernel(const typename Tr::elem* logits, int64_t row_stride,
                                                                        int32_t V, typename Tr::elem* dlogits,
                                                                        ClusterArgs a, int32_t vpt,
                                                                        const float* __restrict__ gcoef)
{
    if (*a.sync_fail == 0u) return;
    constexpr int E = Tr::kPerVec;
    constexpr int NT = kClusterThreads;
    const int C = a.C;
    const int nvec = V / E;
    const int tid = threadIdx.x;
    for (int64_t q = blockIdx.x; q < a.N * C; q += gridDim.x) {
        const int64_t row = q / C;
        const int c = (int)(q - row * C);
        if ((a.slots[q * 2 + 1] >> 32) != kTagPending || a.f.defer[row] != 0) continue;   // uniform over the workgroup
        const float g = gcoef[row] * a.f.grad_out;
        const float l = a.f.lse[row];
        const int32_t y = a.f.token_ids[row];
        const bool live = row_is_live(g, l, y, V);
        const typename Tr::elem* rowp = logits + row * row_stride;
        typename Tr::elem* outp = dlogits + row * row_stride;
        const float cexp = live ? fmaf(-l, kLog2e, log2f(fabsf(g))) : 0.0f;
        const bool negate = g > 0.0f;
        const float sgn = negate ? -1.0f : 1.0f;
        const float g_mag = negate ? -g : g;
        const int yvec = y / E;
        const int first = c * NT * vpt;
        for (int k = 0; k < vpt; ++k) {
            const int i = first + k * NT + tid;
            if (i >= nvec) break;
            u32x4* op = reinterpret_cast<u32x4*>(outp) + i;
            if (!live) {
                store_stream(op, u32x4{0u, 0u, 0u, 0u});
                continue;
            }
            float f[E];
            Tr::unpack(load_stream(reinterpret_cast<const u32x4*>(rowp) + i), f);
#pragma unroll
            for (int e = 0; e < E; ++e) f[e] = fast_exp2(fmaf(f[e], kLog2e, cexp));
            if (i == yvec) {
#pragma unroll
                for (int e = 0; e < E; ++e) f[e] += (e == y - yvec * E) ? g_mag : 0.0f;
            }
            u32x4 o = Tr::pack(f);
            if (negate) o ^= Tr::sign_bits();
            store_stream(op, o);
        }
        if (c == C - 1 && tid == NT - 1) {      // ragged tail of the row
            for (int j = nvec * E; j < V; ++j) {
                float x = 0.0f;
                if (live) {
                    x = sgn * fast_exp2(fmaf(Tr::load1(rowp + j), kLog2e, cexp));
                    if (j == y) x += g;
                }
                Tr::store1(outp + j, x);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// forward call by pieces: the statistics half of the row-cooperative kernel
// ---------------------------------------------------------------------------------------------
// The same pieces, the same per-piece arithmetic and the same merge tree as cluster_row_kernel, so
// lse, log-prob and entropy (and every decision taken from them) carry the same bits on both paths.
// No waiting here: a second kernel merges the pieces.  Consecutive workgroups read consecutive
// 61 KB pieces, the access pattern HBM serves best.
template <class Tr, int VPT>
__global__ __launch_bounds__(kClusterThreads) void piece_stats_kernel(const typename Tr::elem* logits, int64_t row_stride,
                                                                      int32_t V, int64_t N, int32_t C,
                                                                      unsigned long long* slots)
{
    constexpr int NT = kClusterThreads;
    constexpr int E = Tr::kPerVec;
    constexpr int P = NT * VPT;
    const int c = blockIdx.x;
    const int64_t row = (int64_t)blockIdx.z * kRowsPerGridY + blockIdx.y;
    if (row >= N) return;
    const int tid = threadIdx.x;
    const typename Tr::elem* rowp = logits + row * row_stride;
    const u32x4* vp = reinterpret_cast<const u32x4*>(rowp);
    const int nvec = V / E;
    const int first = c * P;
    const bool full = first + P <= nvec;
    const bool owns_tail = (c == C - 1) && (tid == NT - 1) && (nvec * E < V);
    u32x4 v[VPT];
    __shared__ float sm[NT / 64], sS[NT / 64], sT[NT / 64];
    float m, S, T;
    piece_statistics<Tr, VPT>(vp, rowp, nvec, V, first, full, owns_tail, v, sm, sS, sT, m, S, T);
    if (tid == 0) {
        unsigned long long* slot = slots + (row * C + c) * 2;
        slot[0] = piece_word0(m, S);
        slot[1] = piece_word1(T);
    }
}

// One wave per row: lane c brings piece c, the tree merges them, lane 0 finishes the row.
template <class Tr>
__global__ __launch_bounds__(256) void piece_merge_kernel(const typename Tr::elem* logits, int64_t row_stride, int32_t V,
                                                          int64_t N, int32_t C, const unsigned long long* slots,
                                                          const int32_t* __restrict__ token_ids,
                                                          float* __restrict__ lse_out, float* __restrict__ logp_out,
                                                          float* __restrict__ ent_out)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= N) return;
    float pm = kEmpty, pS = 0.0f, pT = 0.0f;
    if (lane < C) {
        const unsigned long long w0 = slots[(row * C + lane) * 2], w1 = slots[(row * C + lane) * 2 + 1];
        pm = __uint_as_float((uint32_t)w0);
        pS = __uint_as_float((uint32_t)(w0 >> 32));
        pT = __uint_as_float((uint32_t)w1);
    }
    merge_pieces_tree(pm, pS, pT);
    if (lane == 0) {
        const int32_t y = token_ids[row];
        const bool has_y = y >= 0 && y < V;
        const float zy = has_y ? Tr::load1(logits + row * row_stride + y) : 0.0f;
        float lse, lp, ent;
        finish_pieces(pm, pS, pT, has_y, zy, lse, lp, ent);
        lse_out[row] = lse;
        logp_out[row] = lp;
        ent_out[row] = ent;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
// Shape of the one-workgroup-per-row kernels (row_stats_kernel, fused_row_kernel): 512 threads,
// eight 16-byte loads in flight per lane.  One shape for both, so that their row statistics are
// bit-identical.
constexpr int kRowThreads = 512;
constexpr int kRowUnroll = 8;

bool shape_ok(int64_t N, int64_t V, int64_t stride)
{
    return N > 0 && N <= kMaxRows && V > 0 && V <= 0x7fffffffLL && stride >= V;
}

int32_t check_logits(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t stride)
{
    if (!logits) return ULORL_ERR_NULL;
    if (dt != ULORL_F32 && dt != ULORL_BF16) return ULORL_ERR_DTYPE;
    if (!shape_ok(N, V, stride)) return ULORL_ERR_SHAPE;
    const size_t esz = dt == ULORL_F32 ? 4 : 2;
    if (((uintptr_t)logits & 15u) != 0 || ((size_t)stride * esz) % 16 != 0) return ULORL_ERR_ALIGN;
    return ULORL_OK;
}

dim3 rows_grid(unsigned x, int64_t N)
{
    return dim3(x, (unsigned)(N < kRowsPerGridY ? N : kRowsPerGridY), (unsigned)((N + kRowsPerGridY - 1) / kRowsPerGridY));
}

template <class Tr>
void launch_row_stats(const void* logits, int64_t N, int64_t V, int64_t stride, const int32_t* y, float* lse,
                      float* logp, float* ent, hipStream_t st)
{
    hipLaunchKernelGGL((row_stats_kernel<Tr, kRowThreads, kRowUnroll>), dim3((unsigned)N), dim3(kRowThreads), 0, st,
                       (const typename Tr::elem*)logits, stride, (int32_t)V, y, lse, logp, ent);
}

template <class Tr>
void launch_dlogits(const void* logits, int64_t N, int64_t V, int64_t stride, const int32_t* y, const float* lse,
                    const float* g, float grad_out, void* dz, hipStream_t st)
{
    const int64_t nvec = V / Tr::kPerVec;
    const int64_t chunks = nvec > 0 ? (nvec + 255) / 256 : 1;      // at most 2^21: V < 2^31
    hipLaunchKernelGGL((dlogits_chunk_kernel<Tr>), rows_grid((unsigned)chunks, N), dim3(256), 0, st,
                       (const typename Tr::elem*)logits, stride, (int32_t)V, N, y, lse, g, grad_out,
                       (typename Tr::elem*)dz);
}

// The gradient of the rows flagged in `defer`, through a compacted list.
template <class Tr>
void launch_dlogits_deferred(const void* logits, int64_t N, int64_t V, int64_t stride, const int32_t* y, const float* lse,
                             const float* g, float grad_out, void* dz, const uint8_t* defer, uint32_t* list,
                             uint32_t* count, hipStream_t st)
{
    const int64_t nvec = V / Tr::kPerVec;
    const int64_t chunks = nvec > 0 ? (nvec + 255) / 256 : 1;
    hipLaunchKernelGGL(defer_compact_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, defer, N, list, count);
    hipLaunchKernelGGL((dlogits_rows_kernel<Tr>), dim3((unsigned)chunks, kListRowSlots), dim3(256), 0, st,
                       (const typename Tr::elem*)logits, stride, (int32_t)V, (const uint32_t*)list, (const uint32_t*)count, y,
                       lse, g, grad_out, (typename Tr::elem*)dz);
}

template <class Tr>
void launch_fused_rows(const void* logits, int64_t N, int64_t V, int64_t stride, void* dz, const FusedArgs& a, hipStream_t st)
{
    hipLaunchKernelGGL((fused_row_kernel<Tr, kRowThreads, kRowUnroll>), dim3((unsigned)N), dim3(kRowThreads), 0, st,
                       (const typename Tr::elem*)logits, stride, (int32_t)V, (typename Tr::elem*)dz, a);
}

template <class Tr>
bool launch_piece_stats(const ClusterShape& shape, const void* logits, int64_t N, int64_t V, int64_t stride,
                        const int32_t* y, float* lse, float* logp, float* ent, unsigned long long* slots, hipStream_t st)
{
    const dim3 grid = rows_grid((unsigned)shape.pieces, N);
    bool launched = false;
#define ULORL_CASE(VPT_)                                                                                        \
    if (shape.vpt == VPT_) {                                                                                    \
        hipLaunchKernelGGL((piece_stats_kernel<Tr, VPT_>), grid, dim3(kClusterThreads), 0, st,                  \
                           (const typename Tr::elem*)logits, stride, (int32_t)V, N, (int32_t)shape.pieces, slots); \
        launched = true;                                                                                        \
    }
    ULORL_CASE(4) ULORL_CASE(8) ULORL_CASE(15)
#undef ULORL_CASE
    if (!launched) return false;
    hipLaunchKernelGGL((piece_merge_kernel<Tr>), dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st,
                       (const typename Tr::elem*)logits, stride, (int32_t)V, N, (int32_t)shape.pieces, slots, y, lse, logp,
                       ent);
    return true;
}

template <class Tr>
bool launch_cluster(int vpt, const void* logits, int64_t N, int64_t V, int64_t stride, void* dz, const ClusterArgs& a,
                    hipStream_t st)
{
    // x: piece (fastest, so a row's pieces have consecutive linear ids and land on different XCDs:
    // putting a row's pieces on one XCD measured 15 % slower), y/z: row
    const dim3 grid = rows_grid((unsigned)a.C, N);
#define ULORL_CASE(VPT_)                                                                                       \
    if (vpt == VPT_) {                                                                                         \
        hipLaunchKernelGGL((cluster_row_kernel<Tr, VPT_>), grid, dim3(kClusterThreads), 0, st,                 \
                           (const typename Tr::elem*)logits, stride, (int32_t)V, (typename Tr::elem*)dz, a);   \
        return true;                                                                                           \
    }
    ULORL_CASE(4) ULORL_CASE(8) ULORL_CASE(15)
#undef ULORL_CASE
    return false;
}

int32_t check_fwd_bwd_args(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
                           const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R, const float* old_logp,
                           const float* advantages, const ulorl_params* p, const float* loss, const float* logp,
                           const float* entropy, const float* lse, const float* gcoef, const void* dlogits)
{
    int32_t rc = check_logits(logits, dt, N, V, row_stride);
    if (rc != ULORL_OK) return rc;
    if (!token_ids || !logp || !entropy || !lse || !advantages || !dlogits) return ULORL_ERR_NULL;
    if (((uintptr_t)dlogits & 15u) != 0) return ULORL_ERR_ALIGN;
    return check_objective_args(cu_seqlens, R, old_logp, p, loss, gcoef);
}

}  // namespace

namespace ulorl_detail {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Shape of the row-cooperative kernel for a row of V elements: vectors per thread and pieces
// (workgroups) per row; pieces == 0 if the row is too long for one wave to poll its pieces.
// A function of V and the storage type only, so the workspace size is too.
ClusterShape cluster_shape(int64_t V, int32_t dt)
{
    const int64_t nvec = V / (dt == ULORL_F32 ? 4 : 8);
    ClusterShape c;
    c.vpt = nvec >= kClusterThreads * 15 ? 15 : nvec >= kClusterThreads * 8 ? 8 : 4;
    const int64_t per_piece = kClusterThreads * (int64_t)c.vpt;
    const int64_t pieces = nvec > 0 ? (nvec + per_piece - 1) / per_piece : 1;
    c.pieces = pieces <= kClusterMaxPieces ? (int)pieces : 0;
    return c;
}

WorkspaceLayout workspace_layout(int64_t N, int64_t V, int32_t R)
{
    WorkspaceLayout w;
    w.nblk = (N + kTokBlock - 1) / kTokBlock;
    // exchange slots of the row-cooperative kernel, sized for the storage type that needs more pieces
    const ClusterShape a = cluster_shape(V, ULORL_F32), b = cluster_shape(V, ULORL_BF16);
    const int pieces = V > 0 ? (a.pieces > b.pieces ? a.pieces : b.pieces) : 0;
    size_t off = 0;
    w.slots = off;    off = align_up(off + sizeof(unsigned long long) * 2 * (size_t)N * (size_t)pieces, 256);   // first: see ulorl_token_loss_fwd
    w.syncfail = off; off = align_up(off + sizeof(uint32_t), 256);
    w.hsum = off;     off = align_up(off + sizeof(double) * (size_t)R, 256);
    w.rflags = off;   off = align_up(off + sizeof(uint32_t) * (size_t)R, 256);
    w.part_sum = off; off = align_up(off + sizeof(double) * (size_t)w.nblk, 256);
    w.part_cnt = off; off = align_up(off + sizeof(int64_t) * 4 * (size_t)w.nblk, 256);
    w.defer = off;    off = align_up(off + (size_t)N, 256);
    w.badcu = off;    off = align_up(off + sizeof(uint32_t), 256);
    w.zy = off;       off = align_up(off + (V > 0 ? sizeof(float) * (size_t)N : 0), 256);
    w.defer_list = off;  off = align_up(off + (V > 0 ? sizeof(uint32_t) * (size_t)N : 0), 256);
    w.defer_count = off; off = align_up(off + sizeof(uint32_t), 256);
    w.total = off;
    return w;
}

int32_t resolve_launch(const ulorl_launch* launch, LaunchOpts* out)
{
    *out = LaunchOpts();
    if (!launch) return ULORL_OK;
    if ((launch->flags & ~(uint32_t)(ULORL_LAUNCH_PER_ROW | ULORL_LAUNCH_DENSE_ROWS)) != 0) return ULORL_ERR_PARAM;
    for (int i = 0; i < 4; ++i)
        if (launch->reserved[i] != 0) return ULORL_ERR_PARAM;
    if (launch->sync_spins < 0 || launch->gemm_tile < 0 || launch->gemm_tile > 1 || launch->gemm_group_m < 0 ||
        launch->gemm_group_m > 64)
        return ULORL_ERR_PARAM;
    out->per_row = (launch->flags & ULORL_LAUNCH_PER_ROW) != 0;
    out->dense_rows = (launch->flags & ULORL_LAUNCH_DENSE_ROWS) != 0;
    if (launch->sync_spins > 0) out->sync_spins = launch->sync_spins;
    out->gemm_tile = launch->gemm_tile;
    if (launch->gemm_group_m > 0) out->gemm_group_m = launch->gemm_group_m;
    return ULORL_OK;
}

int32_t resolve_segment_stats(const ulorl_segment_stats* st, int64_t N, SegStatsArgs* out)
{
    *out = SegStatsArgs();
    out->K = 0;
    if (!st) return ULORL_OK;
    if (st->K <= 0 || st->K > kSegMaxK || st->reserved != 0 || N > 0x7fffffffLL) return ULORL_ERR_SHAPE;
    if (!st->count || !st->ratio_sum || !st->ratio_max || !st->clipped || !st->kl_sum || !st->ent_sum || !st->masked)
        return ULORL_ERR_NULL;
    if (!st->workspace || ((uintptr_t)st->workspace & 255u) != 0 || st->workspace_bytes < seg_workspace_bytes(N, st->K))
        return ULORL_ERR_WORKSPACE;
    const size_t nblk = (size_t)((N + kSegBlock - 1) / kSegBlock);
    out->K = st->K;
    out->part = (double*)st->workspace;
    out->part_oor = (double*)((char*)st->workspace + seg_align_up(nblk * (size_t)st->K * kSegStats * sizeof(double), 256));
    out->count = st->count; out->ratio_sum = st->ratio_sum; out->ratio_max = st->ratio_max;
    out->clipped = st->clipped; out->kl_sum = st->kl_sum; out->ent_sum = st->ent_sum; out->masked = st->masked;
    out->out_of_range = st->out_of_range;
    return ULORL_OK;
}

// Argument checks shared by the forward and the fused forward+backward entry points.
int32_t check_objective_args(const int32_t* cu_seqlens, int32_t R, const float* old_logp, const ulorl_params* p,
                             const float* loss, const float* gcoef)
{
    if (!p || !cu_seqlens || !loss || !gcoef) return ULORL_ERR_NULL;
    if (R <= 0) return ULORL_ERR_SHAPE;
    if (!(p->eps_low >= 0.0f) || !(p->eps_high >= 0.0f) || !(p->tau > 0.0f && p->tau <= 1.0f) ||
        !(p->sigma == p->sigma) || p->seg_len < 0 || p->reserved != 0)
        return ULORL_ERR_PARAM;
    if (p->is_mode != ULORL_IS_SAIS && p->is_mode != ULORL_IS_POIS) return ULORL_ERR_PARAM;
    if (p->gate_mode < ULORL_GATE_PER_RESPONSE || p->gate_mode > ULORL_GATE_NEVER) return ULORL_ERR_PARAM;
    if (p->is_mode == ULORL_IS_SAIS && !old_logp) return ULORL_ERR_NULL;
    return ULORL_OK;
}

TokenArgs make_token_args(int64_t N, int64_t V, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R,
                          const int32_t* segment_ids, const float* old_logp, const float* advantages,
                          const ulorl_params* p, float* logp, float* entropy, float* lse, float* gcoef,
                          uint8_t* mpt_mask, float* ratio, int32_t* segment_out, float* resp_entropy,
                          uint8_t* resp_gate, void* workspace, const WorkspaceLayout& wl, const SegStatsArgs& seg)
{
    char* ws = (char*)workspace;
    TokenArgs a;
    a.logp = logp; a.entropy = entropy; a.lse = lse; a.token_ids = token_ids; a.cu = cu_seqlens;
    a.segment_ids = segment_ids; a.old_logp = old_logp; a.adv = advantages;
    a.gcoef = gcoef;
    a.mask = mpt_mask; a.ratio = ratio; a.seg_out = segment_out; a.resp_entropy = resp_entropy;
    a.resp_gate = resp_gate;
    a.hsum = (double*)(ws + wl.hsum); a.rflags = (uint32_t*)(ws + wl.rflags);
    a.sync_fail = nullptr;
    a.part_sum = (double*)(ws + wl.part_sum); a.part_cnt = (int64_t*)(ws + wl.part_cnt);
    a.N = N; a.V = (int32_t)V; a.R = R;
    a.is_mode = p->is_mode; a.gate_mode = p->gate_mode; a.seg_len = p->seg_len;
    a.eps_low = (double)p->eps_low; a.eps_high = (double)p->eps_high;
    a.tau = (double)p->tau; a.sigma = (double)p->sigma;
    a.D = p->denominator > 0.0 ? p->denominator : (double)N;
    a.log_tau = log(a.tau);
    a.inv_D = 1.0 / a.D;
    a.seg = seg;
    return a;
}

void launch_token_epilogue(const TokenArgs& a, const WorkspaceLayout& wl, float* loss, int64_t* counters, hipStream_t st)
{
    const size_t seg_lds = (size_t)a.seg.K * kSegStats * sizeof(double);
    hipLaunchKernelGGL(response_entropy_kernel, dim3((unsigned)a.R), dim3(kTokBlock), 0, st, a);
    hipLaunchKernelGGL(token_terms_kernel, dim3((unsigned)wl.nblk), dim3(kTokBlock), seg_lds, st, a);
    hipLaunchKernelGGL(loss_finalize_kernel, dim3(1), dim3(kTokBlock), 0, st, a, wl.nblk, loss, counters);
}

}  // namespace ulorl_detail

// Scratch memory of ulorl_token_loss_fwd_bwd_static, the entry point for callers that cannot
// allocate: the workspace of the one-call path (exchange slots, per-response sums, per-block
// partial sums, nine bytes per row) in a file-scope device array.  Every GPU the library runs
// on holds its own copy until the process ends.  The name below is a host-side stand-in, never a
// device address: host code uses the pointer static_scratch_for_current_device() resolves.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Address of this device's copy of the static scratch array, resolved once per device (each GPU
// holds its own copy of a __device__ array at its own address).
int32_t static_scratch_for_current_device(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ULORL_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (ptrs[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return ULORL_ERR_HIP;
        if (((uintptr_t)ptr & 255u) != 0) return ULORL_ERR_HIP;
        ptrs[dev] = ptr;
    }
    *out = ptrs[dev];
    return ULORL_OK;
}

// The one-call path on a validated problem and a workspace of at least wl.total bytes.
int32_t fwd_bwd_enqueue(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
                        const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R, const int32_t* segment_ids,
                        const float* old_logp, const float* advantages, const ulorl_params* p, float grad_out,
                        float* loss, float* logp, float* entropy, float* lse, float* gcoef, uint8_t* mpt_mask,
                        float* ratio, int32_t* segment_out, float* resp_entropy, uint8_t* resp_gate,
                        int64_t* counters, const SegStatsArgs& seg, void* dlogits, void* workspace,
                        const WorkspaceLayout& wl, const LaunchOpts& opts, void* hip_stream)
{
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const bool bf16 = dt == ULORL_BF16;

    TokenArgs a = make_token_args(N, V, token_ids, cu_seqlens, R, segment_ids, old_logp, advantages, p, logp, entropy,
                                  lse, gcoef, mpt_mask, ratio, segment_out, resp_entropy, resp_gate, workspace, wl, seg);
    FusedArgs f;
    f.token_ids = token_ids; f.old_logp = old_logp; f.adv = advantages;
    f.lse = lse; f.logp = logp; f.entropy = entropy;
    f.defer = (uint8_t*)(ws + wl.defer); f.zy_row = (float*)(ws + wl.zy); f.badcu = (const uint32_t*)(ws + wl.badcu);
    f.is_mode = a.is_mode; f.gate_mode = a.gate_mode;
    f.eps_low = a.eps_low; f.eps_high = a.eps_high; f.log_tau = a.log_tau; f.inv_D = a.inv_D;
    f.grad_out = grad_out;

    hipLaunchKernelGGL(cu_check_kernel, dim3(1), dim3(kTokBlock), 0, st, cu_seqlens, R, N, (uint32_t*)(ws + wl.badcu),
                       (uint32_t*)(ws + wl.defer_count));
    const ClusterShape shape = cluster_shape(V, dt);
    const bool cooperative = !opts.per_row && shape.pieces > 0 && 2 * N * (int64_t)shape.pieces < (1LL << 38);
    ClusterArgs ca = {};
    if (cooperative) {
        ca.f = f;
        ca.slots = (unsigned long long*)(ws + wl.slots);
        ca.sync_fail = (uint32_t*)(ws + wl.syncfail);
        ca.N = N;
        ca.C = shape.pieces;
        ca.spin_limit = opts.sync_spins;
        a.sync_fail = ca.sync_fail;
        const int64_t nslots = 2 * N * (int64_t)shape.pieces;
        hipLaunchKernelGGL(fill_zero_u64_kernel, dim3((unsigned)((nslots + 255) / 256)), dim3(256), 0, st, ca.slots, nslots,
                           ca.sync_fail);
        const bool ok = bf16 ? launch_cluster<StoreBF16>(shape.vpt, logits, N, V, row_stride, dlogits, ca, st)
                             : launch_cluster<StoreF32>(shape.vpt, logits, N, V, row_stride, dlogits, ca, st);
        if (!ok) return ULORL_ERR_HIP;
        hipLaunchKernelGGL(repair_rows_kernel, dim3(kRepairRowGrid), dim3(256), 0, st, ca, (int32_t)V);
    } else if (bf16) {
        launch_fused_rows<StoreBF16>(logits, N, V, row_stride, dlogits, f, st);
    } else {
        launch_fused_rows<StoreF32>(logits, N, V, row_stride, dlogits, f, st);
    }
    if (hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;
    launch_token_epilogue(a, wl, loss, counters, st);
    if (hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;
    if (a.gate_mode == ULORL_GATE_PER_RESPONSE || a.gate_mode == ULORL_GATE_GLOBAL) {
        // MPT members waited for the gate: their rows are still logits (in place) or unwritten
        uint32_t* list = (uint32_t*)(ws + wl.defer_list);
        uint32_t* count = (uint32_t*)(ws + wl.defer_count);
        if (bf16)
            launch_dlogits_deferred<StoreBF16>(logits, N, V, row_stride, token_ids, lse, gcoef, grad_out, dlogits, f.defer, list,
                                               count, st);
        else
            launch_dlogits_deferred<StoreF32>(logits, N, V, row_stride, token_ids, lse, gcoef, grad_out, dlogits, f.defer, list,
                                              count, st);
    }
    if (cooperative) {
        if (bf16)
            hipLaunchKernelGGL((repair_pieces_kernel<StoreBF16>), dim3(kRepairPieceGrid), dim3(kClusterThreads), 0, st,
                               (const uint16_t*)logits, row_stride, (int32_t)V, (uint16_t*)dlogits, ca, (int32_t)shape.vpt,
                               (const float*)gcoef);
        else
            hipLaunchKernelGGL((repair_pieces_kernel<StoreF32>), dim3(kRepairPieceGrid), dim3(kClusterThreads), 0, st,
                               (const float*)logits, row_stride, (int32_t)V, (float*)dlogits, ca, (int32_t)shape.vpt,
                               (const float*)gcoef);
    }
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

}  // namespace

extern "C" {

int32_t ulorl_version(void) { return 200; }

const char* ulorl_status_string(int32_t status)
{
    switch (status) {
    case ULORL_OK: return "ok";
    case ULORL_ERR_NULL: return "required pointer is NULL";
    case ULORL_ERR_SHAPE: return "shape out of range";
    case ULORL_ERR_DTYPE: return "unknown storage type";
    case ULORL_ERR_ALIGN: return "logits base or row stride not 16-byte aligned";
    case ULORL_ERR_PARAM: return "invalid parameter";
    case ULORL_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ULORL_ERR_HIP: return "HIP launch failed";
    case ULORL_ERR_TOO_LARGE: return "problem needs more scratch memory than the static array holds";
    default: return "unknown status";
    }
}

size_t ulorl_token_loss_workspace_bytes(int64_t N, int64_t V, int32_t R)
{
    if (N <= 0 || N > kMaxRows || V <= 0 || V > 0x7fffffffLL || R <= 0) return 0;
    return workspace_layout(N, V, R).total;
}

int32_t ulorl_token_loss_fwd(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
                             const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R,
                             const int32_t* segment_ids, const float* old_logp, const float* advantages,
                             const ulorl_params* p, float* loss, float* logp, float* entropy, float* lse,
                             float* gcoef, uint8_t* mpt_mask, float* ratio, int32_t* segment_out,
                             float* resp_entropy, uint8_t* resp_gate, int64_t* counters,
                             const ulorl_segment_stats* seg_stats, void* workspace, size_t workspace_bytes,
                             const ulorl_launch* launch, void* hip_stream)
{
    int32_t rc = check_logits(logits, dt, N, V, row_stride);
    if (rc != ULORL_OK) return rc;
    if (!token_ids || !logp || !entropy || !lse) return ULORL_ERR_NULL;
    LaunchOpts opts;
    rc = resolve_launch(launch, &opts);
    if (rc != ULORL_OK) return rc;
    const bool stats_only = advantages == nullptr;
    WorkspaceLayout wl = {};
    SegStatsArgs seg;
    seg.K = 0;
    if (!stats_only) {
        rc = check_objective_args(cu_seqlens, R, old_logp, p, loss, gcoef);
        if (rc != ULORL_OK) return rc;
        rc = resolve_segment_stats(seg_stats, N, &seg);
        if (rc != ULORL_OK) return rc;
        wl = workspace_layout(N, V, R);
        if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < wl.total)
            return ULORL_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)hip_stream;

    // Statistics by pieces (the row-cooperative kernel's first half, bit-identical with it) when the
    // caller gave a workspace that holds the pieces' slots; else one looping workgroup per row.
    const ClusterShape shape = cluster_shape(V, dt);
    const size_t slot_bytes = sizeof(unsigned long long) * 2 * (size_t)N * (size_t)(shape.pieces > 0 ? shape.pieces : 0);
    const bool by_pieces = !opts.per_row && shape.pieces > 0 && workspace != nullptr &&
                           ((uintptr_t)workspace & 255u) == 0 && workspace_bytes >= slot_bytes;
    if (by_pieces) {
        unsigned long long* slots = (unsigned long long*)workspace;    // the layout's first region
        const bool ok = dt == ULORL_BF16
                 ? launch_piece_stats<StoreBF16>(shape, logits, N, V, row_stride, token_ids, lse, logp, entropy, slots, st)
                 : launch_piece_stats<StoreF32>(shape, logits, N, V, row_stride, token_ids, lse, logp, entropy, slots, st);
        if (!ok) return ULORL_ERR_HIP;
    } else if (dt == ULORL_BF16) {
        launch_row_stats<StoreBF16>(logits, N, V, row_stride, token_ids, lse, logp, entropy, st);
    } else {
        launch_row_stats<StoreF32>(logits, N, V, row_stride, token_ids, lse, logp, entropy, st);
    }
    if (hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;
    if (stats_only) return ULORL_OK;

    const TokenArgs a = make_token_args(N, V, token_ids, cu_seqlens, R, segment_ids, old_logp, advantages, p, logp,
                                        entropy, lse, gcoef, mpt_mask, ratio, segment_out, resp_entropy, resp_gate,
                                        workspace, wl, seg);
    launch_token_epilogue(a, wl, loss, counters, st);
    if (hipGetLastError() != hipSuccess) return ULORL_ERR_HIP;
    return ULORL_OK;
}

int32_t ulorl_token_loss_fwd_bwd(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
                                 const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R,
                                 const int32_t* segment_ids, const float* old_logp, const float* advantages,
                                 const ulorl_params* p, float grad_out, float* loss, float* logp, float* entropy,
                                 float* lse, float* gcoef, uint8_t* mpt_mask, float* ratio, int32_t* segment_out,
                                 float* resp_entropy, uint8_t* resp_gate, int64_t* counters,
                                 const ulorl_segment_stats* seg_stats, void* dlogits, void* workspace,
                                 size_t workspace_bytes, const ulorl_launch* launch, void* hip_stream)
{
    int32_t rc = check_fwd_bwd_args(logits, dt, N, V, row_stride, token_ids, cu_seqlens, R, old_logp, advantages, p,
                                    loss, logp, entropy, lse, gcoef, dlogits);
    if (rc != ULORL_OK) return rc;
    LaunchOpts opts;
    rc = resolve_launch(launch, &opts);
    if (rc != ULORL_OK) return rc;
    SegStatsArgs seg;
    rc = resolve_segment_stats(seg_stats, N, &seg);
    if (rc != ULORL_OK) return rc;
    const WorkspaceLayout wl = workspace_layout(N, V, R);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < wl.total) return ULORL_ERR_WORKSPACE;
    return fwd_bwd_enqueue(logits, dt, N, V, row_stride, token_ids, cu_seqlens, R, segment_ids, old_logp, advantages, p,
                           grad_out, loss, logp, entropy, lse, gcoef, mpt_mask, ratio, segment_out, resp_entropy,
                           resp_gate, counters, seg, dlogits, workspace, wl, opts, hip_stream);
}

int32_t ulorl_init(void)
{
    void* ptr = nullptr;
    return static_scratch_for_current_device(&ptr);
}

size_t ulorl_static_scratch_bytes(void) { return kStaticScratchBytes; }

int32_t ulorl_token_loss_fwd_bwd_static(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
                                        const int32_t* token_ids, const int32_t* cu_seqlens, int32_t R,
                                        const int32_t* segment_ids, const float* old_logp, const float* advantages,
                                        const ulorl_params* p, float grad_out, float* loss, float* logp,
                                        float* entropy, float* lse, float* gcoef, uint8_t* mpt_mask, float* ratio,
                                        int32_t* segment_out, float* resp_entropy, uint8_t* resp_gate,
                                        int64_t* counters, const ulorl_segment_stats* seg_stats, void* dlogits,
                                        const ulorl_launch* launch, void* hip_stream)
{
    int32_t rc = check_fwd_bwd_args(logits, dt, N, V, row_stride, token_ids, cu_seqlens, R, old_logp, advantages, p,
                                    loss, logp, entropy, lse, gcoef, dlogits);
    if (rc != ULORL_OK) return rc;
    LaunchOpts opts;
    rc = resolve_launch(launch, &opts);
    if (rc != ULORL_OK) return rc;
    SegStatsArgs seg;
    rc = resolve_segment_stats(seg_stats, N, &seg);
    if (rc != ULORL_OK) return rc;
    const WorkspaceLayout wl = workspace_layout(N, V, R);
    if (wl.total > kStaticScratchBytes) return ULORL_ERR_TOO_LARGE;
    void* ws = nullptr;
    rc = static_scratch_for_current_device(&ws);
    if (rc != ULORL_OK) return rc;
    return fwd_bwd_enqueue(logits, dt, N, V, row_stride, token_ids, cu_seqlens, R, segment_ids, old_logp, advantages, p,
                           grad_out, loss, logp, entropy, lse, gcoef, mpt_mask, ratio, segment_out, resp_entropy,
                           resp_gate, counters, seg, dlogits, ws, wl, opts, hip_stream);
}

int32_t ulorl_token_loss_bwd(const void* logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
                             const int32_t* token_ids, const float* lse, const float* gcoef, float grad_out,
                             void* dlogits, void* hip_stream)
{
    int32_t rc = check_logits(logits, dt, N, V, row_stride);
    if (rc != ULORL_OK) return rc;
    if (!token_ids || !lse || !gcoef || !dlogits) return ULORL_ERR_NULL;
    if (((uintptr_t)dlogits & 15u) != 0) return ULORL_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    if (dt == ULORL_BF16)
        launch_dlogits<StoreBF16>(logits, N, V, row_stride, token_ids, lse, gcoef, grad_out, dlogits, st);
    else
        launch_dlogits<StoreF32>(logits, N, V, row_stride, token_ids, lse, gcoef, grad_out, dlogits, st);
    return hipGetLastError() == hipSuccess ? ULORL_OK : ULORL_ERR_HIP;
}

}  // extern "C"
