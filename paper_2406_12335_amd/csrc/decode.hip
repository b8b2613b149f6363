// One decode step of the accumulated attention score (paper Eq. 2, taken incrementally;
// order of operations as in Fig. 2): append the new token's row, let its query attend
// over every cached row, add the attention weights to the rows' running scores.
//
// HBM-bound GEMV: every K row is read exactly once, 16 bytes per lane, a group of lanes per
// row.  A (batch, head) unit is split into chunks of kDecodeChunk rows, one workgroup each,
// so that a single sequence still fills the chip.  Each workgroup leaves its logits and its
// chunk's (max, sum of exponentials) in the workspace; the workgroup that finishes last for a
// unit (a per-unit arrival counter, no waiting) combines the chunk statistics and applies
// S += softmax.  Logits live in the base-2 domain: t = c*log2(e)*<q,k>.
#include "vatp_device.h"

namespace vatp {

namespace {

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_score_kernel(
    const T *__restrict__ q, const T *__restrict__ k_new, const T *__restrict__ v_new,
    T *__restrict__ K, T *__restrict__ V, float *__restrict__ S, float *__restrict__ nrm,
    int32_t *__restrict__ pos, float *ws_logit, float2 *ws_part,
    unsigned *__restrict__ counters, BatchMeta meta, int n_heads, int cap, int chunks_alloc,
    float scale_log2)
{
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = 256 / kLanesPerRow;

    __shared__ float s_logit[kDecodeChunk];
    __shared__ float s_red[8];
    __shared__ int s_last;

    const int b = blockIdx.z, h = blockIdx.y, chunk = blockIdx.x;
    const int n0 = meta.len[b];            // rows cached before this step; new row index
    const int n = n0 + 1;
    const int row0 = chunk * kDecodeChunk;
    if (row0 >= n) return;
    const int n_chunks = (n + kDecodeChunk - 1) / kDecodeChunk;
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
    float *logit_u = ws_logit + unit * cap;
    const int sub = threadIdx.x % kLanesPerRow;
    const int rloc = threadIdx.x / kLanesPerRow;

    // this lane's slice of the query, widened once
    float qf[kE];
    Elt<T>::unpack(reinterpret_cast<const uint4 *>(q + unit * D)[sub], qf);

    // the workgroup that owns the new row stores k, v, |v|_1 and pos into the caches
    if (n0 >= row0 && n0 < row0 + kDecodeChunk && threadIdx.x < kLanesPerRow) {
        const uint4 kraw = reinterpret_cast<const uint4 *>(k_new + unit * D)[sub];
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

#pragma unroll
    for (int pass = 0; pass < kDecodeChunk / kRowsPerPass; ++pass) {
        const int rl = pass * kRowsPerPass + rloc;
        const int r = row0 + rl;
        float dot = 0.f;
        if (r < n) {
            // the new row is taken from the step's input, not from the cache being written
            const uint4 raw = (r == n0) ? reinterpret_cast<const uint4 *>(k_new + unit * D)[sub]
                                        : Ku[static_cast<size_t>(r) * kLanesPerRow + sub];
            float kf[kE];
            Elt<T>::unpack(raw, kf);
#pragma unroll
            for (int e = 0; e < kE; ++e) dot = fmaf(qf[e], kf[e], dot);
        }
#pragma unroll
        for (int off = kLanesPerRow / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
        if (sub == 0) s_logit[rl] = (r < n) ? dot * scale_log2 : -INFINITY;
    }
    __syncthreads();

    // chunk statistics: maximum and sum of 2^(t - max) over the chunk's rows
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float t = (threadIdx.x < kDecodeChunk) ? s_logit[threadIdx.x] : -INFINITY;
    float mx = t;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) s_red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    float e = (threadIdx.x < kDecodeChunk) ? exp2f(t - mx) : 0.f;   // 2^(-inf) = 0 for the tail
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) e += __shfl_xor(e, off);
    if (lane == 0) s_red[4 + wave] = e;
    if (threadIdx.x < kDecodeChunk && row0 + threadIdx.x < n) logit_u[row0 + threadIdx.x] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        ws_part[unit * chunks_alloc + chunk] = make_float2(mx, s_red[4] + s_red[5] + s_red[6] + s_red[7]);
    }

    // arrival counter: the last workgroup of the unit finishes the softmax
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned prev = atomicAdd(&counters[unit], 1u);
        s_last = (prev == static_cast<unsigned>(n_chunks - 1));
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();

    float M = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, ws_part[unit * chunks_alloc + c].x);
    float Lsum = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float pm = ws_part[unit * chunks_alloc + c].x;
        const float pl = ws_part[unit * chunks_alloc + c].y;
        Lsum += pl * exp2f(pm - M);
    }
    const float lse2 = M + log2f(Lsum);
    float *Su = S + unit * cap;
    for (int r = threadIdx.x; r < n; r += 256) {
        const float a = exp2f(logit_u[r] - lse2);
        Su[r] = (r == n0 ? 0.f : Su[r]) + a;
    }
    if (threadIdx.x == 0) counters[unit] = 0u;     // leave the counter ready for the next call
}

}  // namespace

hipError_t launch_decode(int dtype, int head_dim, const void *q, const void *k, const void *v,
                         void *K, void *V, float *S, float *nrm, int32_t *pos,
                         float *ws_logit, float2 *ws_part, unsigned *counters,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    const int chunks_alloc = (g.cap + kDecodeChunk - 1) / kDecodeChunk;
    dim3 grid((g.max_len + kDecodeChunk - 1) / kDecodeChunk, g.n_heads, g.batch), block(256);
#define VATP_DEC(T, D)                                                                          \
    hipLaunchKernelGGL((decode_score_kernel<T, D>), grid, block, 0, st,                         \
                       static_cast<const T *>(q), static_cast<const T *>(k),                    \
                       static_cast<const T *>(v), static_cast<T *>(K), static_cast<T *>(V), S,  \
                       nrm, pos, ws_logit, ws_part, counters, meta, g.n_heads, g.cap,           \
                       chunks_alloc, g.scale_log2)
    if (dtype == VATP_F32 && head_dim == 64) VATP_DEC(float, 64);
    else if (dtype == VATP_F32) VATP_DEC(float, 128);
    else if (head_dim == 64) VATP_DEC(bf16_t, 64);
    else VATP_DEC(bf16_t, 128);
#undef VATP_DEC
    return hipGetLastError();
}

}  // namespace vatp
