// Internal declarations shared by the HIP sources of libvatp (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "vatp.h"

namespace vatp {

typedef uint16_t bf16_t;   // raw bfloat16 bits

// Per-sequence host facts, passed to kernels by value (lives in the kernarg segment, 2 KiB of the 4 KiB a
// launch may carry, read with scalar loads): no device copy, no sync.
struct BatchMeta {
    int32_t len[VATP_MAX_BATCH];   // rows valid per sequence on entry
    int32_t aux[VATP_MAX_BATCH];   // budget (select/compact) or new_pos (decode)
};

struct BudgetList {                // the third per-sequence fact of the one-launch decode-and-evict kernel
    int32_t v[VATP_MAX_BATCH];
};

struct Geometry {
    int32_t batch, n_heads, cap, cap_out;
    int32_t n_sink, recent;
    float   scale_log2;            // c * log2(e): logits are kept in the base-2 domain
    int32_t max_len;               // max over the batch of len (decode: len + 1)
    int32_t norm;                  // VATP_NORM_*: value-row norm of the importance (paper Eq. 4, Table 2)
    int32_t group;                 // g >= 1: query heads per K/V head (n_heads counts K/V heads)
    int32_t stream;                // != 0: the call's cache rows exceed what stays resident between steps
};

// A call streams (non-temporal accesses) when the K and V rows it may touch exceed a quarter of the 256 MB
// last-level cache: such a working set cannot survive until the next step of the same layer anyway.
inline bool stream_rows(size_t units, size_t rows, size_t row_bytes) { return units * rows * row_bytes * 2 > (64u << 20); }

// Value-row norm in three steps: lane-local accumulation, combination across the row's lanes,
// final map.  l1 (the paper's metric), l2 and l-infinity (its ablation, Table 2).
__device__ __forceinline__ float norm_accum(int kind, float acc, float x) {
    return kind == VATP_NORM_L1 ? acc + fabsf(x) : kind == VATP_NORM_L2 ? fmaf(x, x, acc) : fmaxf(acc, fabsf(x));
}
__device__ __forceinline__ float norm_combine(int kind, float a, float b) {
    return kind == VATP_NORM_LINF ? fmaxf(a, b) : a + b;
}
__device__ __forceinline__ float norm_finish(int kind, float a) {
    return kind == VATP_NORM_L2 ? sqrtf(a) : kind == VATP_NORM_NONE ? 1.f : a;     // NONE: attention-only baseline
}

// History-window scores (paper Eq. 3: only the attention a token received in the last w+1 steps
// counts) for the fused decode-and-evict step.  hist keeps the last steps' attention weights,
// rows = w + 2 ring rows of cap_hist columns per head: step t writes ring row t mod rows and
// subtracts ring row (t+1) mod rows, which holds step t-w-1.  A cached row owns one column for
// as long as it lives (its `hid`, moved with the row like pos), so evictions never move history:
// the new row takes the column the last evicted row gave up (free_in), or the next fresh one.
// hist == nullptr switches all of this off (accumulated scores, Eq. 2).
struct WindowArgs {
    const float *s_lo;               // [units, cap]      low-order part of every row's score (see window_update)
    float *s_lo_out;                 // [units, cap_out]  ... of the other set
    float *hist;                     // [units, rows, cap_hist]
    int32_t *hid;                    // [units, cap]      column of every row of the current set
    int32_t *hid_out;                // [units, cap_out]  ... of the other set
    const int32_t *free_in;          // [units]           column for the row appended by this step
    int32_t *free_out;               // [units]           ... by the next step
    int32_t rows, cap_hist;
    int32_t step[VATP_MAX_BATCH];    // index t of the new token in its sequence
};

// A windowed score is kept as an unevaluated sum hi + lo of two floats (hi is what S holds): weights enter the
// window and, w+1 steps later, the very same float leaves it, so a sum that is carried exactly stays a sum of
// the weights currently in the window -- its error does not grow with the number of steps, and stays relative
// to the score itself however large the score once was.  Every addition is an error-free transformation (the
// rounding error of hi + x is recovered exactly and folded into lo); what is lost per step is at most 2^-47 of
// the running sum.
__device__ __forceinline__ void two_float_add(float &hi, float &lo, float x)
{
    const float s = __fadd_rn(hi, x);
    const float bb = __fsub_rn(s, hi);
    const float err = __fadd_rn(__fsub_rn(hi, __fsub_rn(s, bb)), __fsub_rn(x, bb));     // hi + x = s + err exactly
    const float l = __fadd_rn(lo, err);
    const float t = __fadd_rn(s, l);                                                   // renormalise: |s| >= |l|
    lo = __fsub_rn(l, __fsub_rn(t, s));
    hi = t;
}
// new score of a windowed row: the weight that leaves the window goes first, then the new one arrives
__device__ __forceinline__ void window_update(float &hi, float &lo, float gone, float p)
{
    two_float_add(hi, lo, -gone);
    two_float_add(hi, lo, p);
    if (hi < 0.f) { hi = 0.f; lo = 0.f; }      // a sum of non-negative terms; its bits are compared as unsigned integers
}

constexpr int kDecodeChunk = 128;  // rows of one unit handled by one workgroup of the decode GEMV

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
    return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

template <typename T> struct Elt;
template <> struct Elt<float> {
    static constexpr int kPer16B = 4;
    __device__ static __forceinline__ void unpack(const uint4 &raw, float *out) {
        out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
        out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
    }
};
template <> struct Elt<bf16_t> {
    static constexpr int kPer16B = 8;
    __device__ static __forceinline__ void unpack(const uint4 &raw, float *out) {
        out[0] = __uint_as_float(raw.x << 16); out[1] = __uint_as_float(raw.x & 0xffff0000u);
        out[2] = __uint_as_float(raw.y << 16); out[3] = __uint_as_float(raw.y & 0xffff0000u);
        out[4] = __uint_as_float(raw.z << 16); out[5] = __uint_as_float(raw.z & 0xffff0000u);
        out[6] = __uint_as_float(raw.w << 16); out[7] = __uint_as_float(raw.w & 0xffff0000u);
    }
};

// ---- streaming accesses ----------------------------------------------------------------------------------
// When one call touches more cache rows than the last-level cache can usefully hold (kStream; chosen by the
// host from the size of the call, see stream_rows), rows are moved with the non-temporal hint: they are read
// once per step and what is written is not read again before the whole model has gone through a step, so the
// lines are not kept in L2 or the last-level cache at the expense of anything else (measured on the fused
// step of 256 heads x 820 rows, 32 layers in turn: 20.4 -> 17.7 us).  Small caches that stay resident from
// one step to the next are accessed the ordinary way (with the hint they ran 5-10 % slower).
typedef unsigned uint4_native __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    const uint4_native x = __builtin_nontemporal_load(reinterpret_cast<const uint4_native *>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void store_stream(uint4 *p, const uint4 &v) {
    const uint4_native x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<uint4_native *>(p));
}

template <bool kStream> __device__ __forceinline__ uint4 load_rows(const uint4 *p) {
    if constexpr (kStream) return load_stream(p); else return *p;
}
template <bool kStream> __device__ __forceinline__ void store_rows(uint4 *p, const uint4 &v) {
    if constexpr (kStream) store_stream(p, v); else *p = v;
}

// ---- reductions across lanes without LDS traffic -----------------------------------------------------------
// Data-parallel-primitive (DPP) operand modifiers move a value between the lanes of a 16-lane row as part of
// a vector-ALU instruction; the shuffles of the HIP headers (ds_bpermute) go through the LDS pipeline instead,
// which a compute unit's 16 wavefronts share.  Lane patterns used: swap within pairs, swap pairs within
// quads, mirror within 8 lanes, mirror within 16 lanes.  Each step combines a lane's value with its partner's
// (both lanes compute the same commutative operation on the same two values), so after step k all lanes of an
// aligned group of 2^k lanes hold identical bits.
template <int kCtrl>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kCtrl, 0xf, 0xf, false));
}
template <int kCtrl>
__device__ __forceinline__ unsigned dpp_move(unsigned x) {
    return static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kCtrl, 0xf, 0xf, false));
}
constexpr int kDppSwapPairs = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppSwapQuadHalves = 0x4E; // quad_perm [2,3,0,1]
constexpr int kDppMirror8 = 0x141;       // row_half_mirror
constexpr int kDppMirror16 = 0x140;      // row_mirror

struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };

// All-reduce over aligned groups of kLanes lanes (a power of two up to 64): every lane of a group ends up with
// the same value.  Groups wider than a 16-lane row finish with one or two LDS-pipeline shuffles.
template <int kLanes, typename Op>
__device__ __forceinline__ float group_all_reduce(float x, Op op)
{
    static_assert(kLanes >= 1 && kLanes <= 64 && (kLanes & (kLanes - 1)) == 0, "group of 1..64 lanes, a power of two");
    if constexpr (kLanes >= 2) x = op(x, dpp_move<kDppSwapPairs>(x));
    if constexpr (kLanes >= 4) x = op(x, dpp_move<kDppSwapQuadHalves>(x));
    if constexpr (kLanes >= 8) x = op(x, dpp_move<kDppMirror8>(x));
    if constexpr (kLanes >= 16) x = op(x, dpp_move<kDppMirror16>(x));
    if constexpr (kLanes >= 32) x = op(x, __shfl_xor(x, 16));
    if constexpr (kLanes >= 64) x = op(x, __shfl_xor(x, 32));
    return x;
}

// All-reduce over the 64 lanes of a wavefront: within the four 16-lane rows by DPP, then the four row results
// are read into scalar registers and combined as (r0 op r1) op (r2 op r3).  The result is wavefront-uniform.
template <typename Op>
__device__ __forceinline__ float wave_all_reduce(float x, Op op)
{
    x = group_all_reduce<16>(x, op);
    const int xi = __builtin_bit_cast(int, x);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 48));
    return op(op(r0, r1), op(r2, r3));
}
__device__ __forceinline__ float wave_sum(float x) { return wave_all_reduce(x, OpSum{}); }
__device__ __forceinline__ float wave_max(float x) { return wave_all_reduce(x, OpMax{}); }

// Workgroup barrier that orders LDS traffic only: every wavefront's LDS operations are complete before any
// wavefront passes, while vector-memory loads that are still in flight stay in flight (__syncthreads would
// wait for them too).  Not a fence for global memory.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Minimum of an unsigned 32-bit key over the wavefront (wavefront-uniform result).
__device__ __forceinline__ unsigned wave_min_u32(unsigned x)
{
    x = min(x, dpp_move<kDppSwapPairs>(x));
    x = min(x, dpp_move<kDppSwapQuadHalves>(x));
    x = min(x, dpp_move<kDppMirror8>(x));
    x = min(x, dpp_move<kDppMirror16>(x));
    const int xi = static_cast<int>(x);
    const unsigned r0 = static_cast<unsigned>(__builtin_amdgcn_readlane(xi, 0)), r1 = static_cast<unsigned>(__builtin_amdgcn_readlane(xi, 16));
    const unsigned r2 = static_cast<unsigned>(__builtin_amdgcn_readlane(xi, 32)), r3 = static_cast<unsigned>(__builtin_amdgcn_readlane(xi, 48));
    return min(min(r0, r1), min(r2, r3));
}

// Minimum of a 64-bit key over the wavefront (same lane patterns; wavefront-uniform result).
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long x)
{
    auto step = [&](auto ctrl) {
        constexpr int kCtrl = decltype(ctrl)::value;
        const unsigned lo = dpp_move<kCtrl>(static_cast<unsigned>(x)), hi = dpp_move<kCtrl>(static_cast<unsigned>(x >> 32));
        const unsigned long long o = (static_cast<unsigned long long>(hi) << 32) | lo;
        x = o < x ? o : x;
    };
    step(std::integral_constant<int, kDppSwapPairs>{});
    step(std::integral_constant<int, kDppSwapQuadHalves>{});
    step(std::integral_constant<int, kDppMirror8>{});
    step(std::integral_constant<int, kDppMirror16>{});
    unsigned long long best = ~0ull;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        const unsigned lo = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<unsigned>(x)), 16 * row));
        const unsigned hi = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<unsigned>(x >> 32)), 16 * row));
        const unsigned long long o = (static_cast<unsigned long long>(hi) << 32) | lo;
        best = o < best ? o : best;
    }
    return best;
}

// This lane's share of <q, k>: the 16 bytes it holds of both rows.  bf16 pairs go through the two-element dot
// instruction (fp32 accumulate), fp32 elements through fused multiply-adds.  Every kernel that forms decode
// logits calls this and then group_all_reduce over the row's lanes, so they all produce the same bits.
template <typename T> __device__ __forceinline__ float dot_16_bytes(const uint4 &k, const uint4 &q);
template <> __device__ __forceinline__ float dot_16_bytes<float>(const uint4 &k, const uint4 &q) {
    float acc = __uint_as_float(k.x) * __uint_as_float(q.x);
    acc = fmaf(__uint_as_float(k.y), __uint_as_float(q.y), acc);
    acc = fmaf(__uint_as_float(k.z), __uint_as_float(q.z), acc);
    return fmaf(__uint_as_float(k.w), __uint_as_float(q.w), acc);
}
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
template <> __device__ __forceinline__ float dot_16_bytes<bf16_t>(const uint4 &k, const uint4 &q) {
    float acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, k.x), __builtin_bit_cast(bf16x2, q.x), 0.f, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, k.y), __builtin_bit_cast(bf16x2, q.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, k.z), __builtin_bit_cast(bf16x2, q.z), acc, false);
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, k.w), __builtin_bit_cast(bf16x2, q.w), acc, false);
}

// Norm of a value row whose 16-byte slices are spread over kLanes lanes (every lane of the group gets it).
template <typename T, int kLanes>
__device__ __forceinline__ float row_norm(int kind, const uint4 &raw)
{
    constexpr int kE = Elt<T>::kPer16B;
    float x[kE], a = 0.f;
    Elt<T>::unpack(raw, x);
#pragma unroll
    for (int e = 0; e < kE; ++e) a = norm_accum(kind, a, x[e]);
    a = kind == VATP_NORM_LINF ? group_all_reduce<kLanes>(a, OpMax{}) : group_all_reduce<kLanes>(a, OpSum{});
    return norm_finish(kind, a);
}

// Softmax statistics of one chunk of kDecodeChunk = 128 logits, formed by ONE wavefront: the lane brings
// logits `lane` and `lane + 64` of the chunk (-inf past the end).  Returns (max, sum of 2^(t - max)): the two
// halves are summed separately and added last.  Every kernel that leaves or uses chunk statistics calls this.
__device__ __forceinline__ float2 chunk_stats_64x2(float t0, float t1)
{
    const float mx = wave_max(fmaxf(t0, t1));
    const float e0 = wave_sum(exp2f(t0 - mx)), e1 = wave_sum(exp2f(t1 - mx));     // 2^(-inf) = 0 past the end
    return make_float2(mx, e0 + e1);
}

// ---- v_mfma_f32_32x32x16_bf16: operand and accumulator conventions shared by the kernels that use it.
// Lane (n = lane & 31, g = lane >> 5) supplies, as A operand, 8 consecutive contraction elements of row n
// of the 32 x 16 left matrix and, as B operand, of column n of the right one (which 8 of the 16 is free as
// long as both operands agree); it receives column n of the 32 x 32 result, rows acc_row(v) + 4 g.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ constexpr int acc_row(int v) { return 8 * (v / 4) + (v % 4); }
// rows of 256 bytes staged in LDS: 16-byte chunk c of row r sits at chunk c ^ (r & 15), so that the 16 lanes
// that read one chunk index of 16 consecutive rows hit 16 different bank groups
__device__ __forceinline__ int swizzled_chunk(int row, int c) { return c ^ (row & 15); }

// Softmax denominator of one decode step from the per-chunk statistics (max_c, sum_c of
// 2^(t - max_c)) that the logits launch left behind: M = max_c max_c and
// L = sum_c sum_c * 2^(max_c - M).  Every wavefront computes both by itself: lanes take chunks
// lane, lane + 64, ... (one round trip to memory, not one per chunk) and combine across the
// wavefront (wave_max / wave_sum), which gives every lane the same bits.  The kernels that finish a decode step all
// call this one function, so they agree bit for bit.
__device__ __forceinline__ void merge_chunk_stats(const float2 *__restrict__ part, int n_chunks, float &M, float &L)
{
    const int lane = threadIdx.x & 63;
    float2 mine = make_float2(-INFINITY, 0.f);
    if (lane < n_chunks) mine = part[lane];
    float m = mine.x;
    for (int c = lane + 64; c < n_chunks; c += 64) m = fmaxf(m, part[c].x);
    m = wave_max(m);
    float l = mine.y * exp2f(mine.x - m);                 // 0 * 2^(-inf) = 0 for lanes without a chunk
    for (int c = lane + 64; c < n_chunks; c += 64) l += part[c].y * exp2f(part[c].x - m);
    M = m;
    L = wave_sum(l);
}

// Component x of the attention output (paper Eq. 1) from the chunks' unnormalised partial sums,
// each relative to its chunk maximum: four independent running sums, so four loads are in flight.
__device__ __forceinline__ float merge_chunk_outputs(const float *__restrict__ ws_out_unit,
                                                     const float2 *__restrict__ part, int n_chunks, int head_dim,
                                                     int x, float M, float L)
{
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < n_chunks; c0 += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u;
            if (c < n_chunks) acc[u] += ws_out_unit[static_cast<size_t>(c) * head_dim + x] * exp2f(part[c].x - M);
        }
    }
    return ((acc[0] + acc[1]) + (acc[2] + acc[3])) / L;
}

// Grouped-query attention: g query heads share a K/V head, each with its own softmax, and a row's
// score grows by the mean of the g attention weights (paper, Limitations section, paragraph on GQA).
// The heads' logits of a unit lie one after the other ([g, cap]), their chunk statistics likewise
// ([g, chunks_alloc]).  lse2[i] = log2 of head i's softmax denominator + log2 g, so that
//     group_weight = sum_i 2^(t_i - lse2[i])
// is that mean.  kMaxG = 1 is plain multi-head attention: the same operations, in the same order,
// as merge_chunk_stats followed by 2^(t - lse2).
template <int kMaxG>
__device__ __forceinline__ void merge_group_stats(const float2 *__restrict__ part, int chunks_alloc, int g,
                                                  int n_chunks, float (&lse2)[kMaxG])
{
    if constexpr (kMaxG == 1) {
        float M, L;
        merge_chunk_stats(part, n_chunks, M, L);
        lse2[0] = M + log2f(L);
    } else {
        const int lane = threadIdx.x & 63;
        float2 mine[kMaxG];
#pragma unroll
        for (int i = 0; i < kMaxG; ++i) {           // every head's first round of loads is in flight at once
            mine[i] = make_float2(-INFINITY, 0.f);
            if (i < g && lane < n_chunks) mine[i] = part[static_cast<size_t>(i) * chunks_alloc + lane];
        }
        const float log2g = log2f(static_cast<float>(g));
#pragma unroll
        for (int i = 0; i < kMaxG; ++i) {
            lse2[i] = 0.f;
            if (i >= g) continue;
            const float2 *pi = part + static_cast<size_t>(i) * chunks_alloc;
            float m = mine[i].x;
            for (int c = lane + 64; c < n_chunks; c += 64) m = fmaxf(m, pi[c].x);
            m = wave_max(m);
            float l = mine[i].y * exp2f(mine[i].x - m);
            for (int c = lane + 64; c < n_chunks; c += 64) l += pi[c].y * exp2f(pi[c].x - m);
            l = wave_sum(l);
            lse2[i] = m + log2f(l) + log2g;
        }
    }
}

// Attention outputs of the new token (paper Eq. 1), one per query head of the unit: thread idx -> (head idx / D,
// component idx % D).  A wavefront works on one head at a time (D is a multiple of 64 or divides it evenly into
// whole heads... D = 64 or 128), so it forms that head's softmax statistics itself, by the same operations as above.
__device__ __forceinline__ void merge_group_outputs(float *__restrict__ out_unit, const float *__restrict__ ws_out_unit,
                                                    const float2 *__restrict__ part, int chunks_alloc, int n_chunks,
                                                    int g, int head_dim, int n_threads)
{
    for (int idx = threadIdx.x; idx < g * head_dim; idx += n_threads) {
        const int i = idx / head_dim, x = idx % head_dim;
        const float2 *pi = part + static_cast<size_t>(i) * chunks_alloc;
        float M, L;
        merge_chunk_stats(pi, n_chunks, M, L);
        out_unit[static_cast<size_t>(i) * head_dim + x] =
            merge_chunk_outputs(ws_out_unit + static_cast<size_t>(i) * chunks_alloc * head_dim, pi, n_chunks, head_dim, x, M, L);
    }
}

// the g logits of row r (head i at Lu + i * cap); zeros when !ok
template <int kMaxG>
__device__ __forceinline__ void load_group_logits(float (&t)[kMaxG], const float *__restrict__ Lu, int cap, int g,
                                                  int r, bool ok)
{
#pragma unroll
    for (int i = 0; i < kMaxG; ++i) t[i] = (ok && i < g) ? Lu[static_cast<size_t>(i) * cap + r] : 0.f;
}

template <int kMaxG>
__device__ __forceinline__ float group_weight(const float (&t)[kMaxG], const float (&lse2)[kMaxG], int g)
{
    float p = exp2f(t[0] - lse2[0]);
#pragma unroll
    for (int i = 1; i < kMaxG; ++i)
        if (i < g) p += exp2f(t[i] - lse2[i]);
    return p;
}

// ---- host-side launchers, one per source file --------------------------------------
hipError_t launch_l1norm(int dtype, int head_dim, const void *V, float *nrm,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

// window >= 0: history-window scores (Eq. 3), the window's attention rows go to hist (may be NULL)
hipError_t launch_prefill_generic(int dtype, int head_dim, const void *Q, const void *K,
                                  float *S, float *lse2, bool have_lse, int window, float *hist,
                                  const BatchMeta &meta, const Geometry &g, hipStream_t st);

hipError_t launch_lse_to_base2(const float *lse, float *lse2, const BatchMeta &meta, const Geometry &g,
                               hipStream_t st);

// (the matrix-core passes also write the value-row norms: no separate launch_l1norm)
// (s_part: room for group * units * cap floats of partial column sums when query heads are grouped, else unused)
hipError_t launch_prefill_mfma(const void *Q, const void *K, const void *V, float *S, float *nrm, float *lse2,
                               float *s_part, bool have_lse, const BatchMeta &meta, const Geometry &g, hipStream_t st);

// history-window prompt scores on the matrix cores (bf16, head_dim 128); lse_part: workspace of
// prefill_window_splits(cap) * units * cap floats; usable if prefill_mfma_window_fits(window, cap, units)
int prefill_window_splits(int cap);
bool prefill_mfma_window_fits(int window, int cap, int n_units);
hipError_t launch_prefill_mfma_window(const void *Q, const void *K, const void *V, float *S, float *nrm, float *lse2,
                                      float *lse_part, int window, float *hist, const BatchMeta &meta,
                                      const Geometry &g, hipStream_t st);

hipError_t launch_decode(int dtype, int head_dim, const void *q, const void *k, const void *v,
                         void *K, void *V, float *S, float *nrm, int32_t *pos,
                         float *ws_logit, float2 *ws_part, float *ws_out, float *out, bool finish,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

// second launch of the fused decode-and-evict step; meta.aux holds the budgets
hipError_t launch_decode_prune(int dtype, int head_dim, const void *K, const void *V, const float *S,
                               const float *nrm, const int32_t *pos, void *K_out, void *V_out, float *S_out,
                               float *nrm_out, int32_t *pos_out, int32_t *kept_idx, const int32_t *synced_in,
                               int32_t *synced_out, const float *ws_logit, const float2 *ws_part,
                               const float *ws_out, float *out, const WindowArgs &win, const BatchMeta &meta,
                               const Geometry &g, hipStream_t st);

// the same step in one launch, one workgroup per head; usable while every head has at most
// decode_prune_one_max_rows() rows after the append
int decode_prune_one_max_rows();
hipError_t launch_decode_prune_one(int dtype, int head_dim, const void *q, const void *k, const void *v, void *K,
                                   void *V, const float *S, float *nrm, int32_t *pos, void *K_out, void *V_out,
                                   float *S_out, float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                                   const int32_t *synced_in, int32_t *synced_out, const BatchMeta &len_pos,
                                   const BudgetList &budget, const Geometry &g, hipStream_t st);

hipError_t launch_select(const float *S, const float *nrm, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

hipError_t launch_gather(int dtype, int head_dim, bool evict_one,
                         const void *K, const void *V, const float *S, const float *nrm,
                         const int32_t *pos, void *K_out, void *V_out, float *S_out,
                         float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

// prompt prune of the history-window variant: columns of the window's attention rows follow kept_idx
// (S_out: the survivors' scores as the selection copied them; s_lo_out receives their low-order parts, such that
// S_out + s_lo_out is the sum of the survivor's window weights carried in two floats)
hipError_t launch_hist_gather(const float *hist_in, const int32_t *kept_idx, float *hist_out, int32_t *hid_out,
                              int32_t *free_out, const float *S_out, float *s_lo_out, int rows, int cap_hist,
                              const BatchMeta &meta, const Geometry &g, hipStream_t st);

}  // namespace vatp
