// One decode step of the accumulated attention score (paper Eq. 2, taken incrementally;
// order of operations as in Fig. 2): append the new token's row, let its query attend
// over every cached row, add the attention weights to the rows' running scores.
//
// HBM-bound GEMV: every K row is read exactly once, 16 bytes per lane, a group of lanes per
// row, four rows in flight per lane.  One workgroup of 1024 threads owns a (batch, head)
// unit, so the softmax over the unit's rows is finished inside the workgroup (LDS and
// wavefront shuffles) and the kernel needs no cross-workgroup hand-off, no atomics and no
// memory fences.  Logits live in the base-2 domain, t = c*log2(e)*<q,k>; they are parked in
// LDS while the unit has at most kLdsRows rows, else in the caller's workspace.
#include "vatp_device.h"

namespace vatp {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kLdsRows = 8192;

__device__ __forceinline__ float block_reduce(float x, bool is_max, float *s_red)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(x, off);
        x = is_max ? fmaxf(x, o) : x + o;
    }
    __syncthreads();                               // s_red may still be read from an earlier call
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = x;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = is_max ? fmaxf(r, s_red[w]) : r + s_red[w];
    return r;
}

template <typename T, int D, bool kLdsLogits>
__global__ __launch_bounds__(kThreads) void decode_score_kernel(
    const T *__restrict__ q, const T *__restrict__ k_new, const T *__restrict__ v_new,
    T *__restrict__ K, T *__restrict__ V, float *__restrict__ S, float *__restrict__ nrm,
    int32_t *__restrict__ pos, float *ws_logit, BatchMeta meta, int n_heads, int cap,
    float scale_log2)
{
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = kThreads / kLanesPerRow;
    constexpr int kUnroll = 4;

    __shared__ float s_logit[kLdsLogits ? kLdsRows : 1];
    __shared__ float s_red[kWaves];

    const size_t unit = blockIdx.x;
    const int b = static_cast<int>(unit / n_heads);
    const int n0 = meta.len[b];            // rows cached before this step = index of the new row
    const int n = n0 + 1;
    const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
    const uint4 *knew = reinterpret_cast<const uint4 *>(k_new + unit * D);
    float *logit = kLdsLogits ? s_logit : ws_logit + unit * cap;
    const int tid = threadIdx.x;
    const int sub = tid % kLanesPerRow;
    const int rloc = tid / kLanesPerRow;

    // this lane's slice of the query, widened once
    float qf[kE];
    Elt<T>::unpack(reinterpret_cast<const uint4 *>(q + unit * D)[sub], qf);

    // append: k, v, |v|_1 and pos of the new token become row n0 of the caches
    if (tid < kLanesPerRow) {
        const uint4 kraw = knew[sub];
        const uint4 vraw = reinterpret_cast<const uint4 *>(v_new + unit * D)[sub];
        reinterpret_cast<uint4 *>(K + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = kraw;
        reinterpret_cast<uint4 *>(V + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = vraw;
        float vf[kE], a = 0.f;
        Elt<T>::unpack(vraw, vf);
#pragma unroll
        for (int e = 0; e < kE; ++e) a += fabsf(vf[e]);
#pragma unroll
        for (int off = kLanesPerRow / 2; off > 0; off >>= 1) a += __shfl_xor(a, off);
        if (sub == 0) {
            nrm[unit * cap + n0] = a;
            if (pos) pos[unit * cap + n0] = meta.aux[b];
        }
    }

    // logits of every row; the new row is read from the step's input, not from the cache
    for (int base = 0; base < n; base += kRowsPerPass * kUnroll) {
        uint4 raw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = base + u * kRowsPerPass + rloc;
            const uint4 *src = (r == n0) ? knew + sub : Ku + static_cast<size_t>(r) * kLanesPerRow + sub;
            raw[u] = (r < n) ? *src : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = base + u * kRowsPerPass + rloc;
            float kf[kE], dot = 0.f;
            Elt<T>::unpack(raw[u], kf);
#pragma unroll
            for (int e = 0; e < kE; ++e) dot = fmaf(qf[e], kf[e], dot);
#pragma unroll
            for (int off = kLanesPerRow / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
            if (sub == 0 && r < n) logit[r] = dot * scale_log2;
        }
    }
    __syncthreads();

    // softmax over the n rows, then S += a
    float mx = -INFINITY;
    for (int r = tid; r < n; r += kThreads) mx = fmaxf(mx, logit[r]);
    mx = block_reduce(mx, true, s_red);
    float sum = 0.f;
    for (int r = tid; r < n; r += kThreads) sum += exp2f(logit[r] - mx);
    sum = block_reduce(sum, false, s_red);
    const float lse2 = mx + log2f(sum);
    float *Su = S + unit * cap;
    for (int r = tid; r < n; r += kThreads) {
        const float a = exp2f(logit[r] - lse2);
        Su[r] = (r == n0 ? 0.f : Su[r]) + a;
    }
}

}  // namespace

hipError_t launch_decode(int dtype, int head_dim, const void *q, const void *k, const void *v,
                         void *K, void *V, float *S, float *nrm, int32_t *pos, float *ws_logit,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    dim3 grid(static_cast<unsigned>(g.batch) * g.n_heads), block(kThreads);
    const bool lds = g.max_len <= kLdsRows;
#define VATP_DEC(T, D, L)                                                                          \
    hipLaunchKernelGGL((decode_score_kernel<T, D, L>), grid, block, 0, st, static_cast<const T *>(q), \
                       static_cast<const T *>(k), static_cast<const T *>(v), static_cast<T *>(K),  \
                       static_cast<T *>(V), S, nrm, pos, ws_logit, meta, g.n_heads, g.cap,         \
                       g.scale_log2)
#define VATP_DEC2(T, D) do { if (lds) VATP_DEC(T, D, true); else VATP_DEC(T, D, false); } while (0)
    if (dtype == VATP_F32 && head_dim == 64) VATP_DEC2(float, 64);
    else if (dtype == VATP_F32) VATP_DEC2(float, 128);
    else if (head_dim == 64) VATP_DEC2(bf16_t, 64);
    else VATP_DEC2(bf16_t, 128);
#undef VATP_DEC2
#undef VATP_DEC
    return hipGetLastError();
}

}  // namespace vatp
