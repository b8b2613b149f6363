// Prompt-pass scoring with plain fp32 FMAs: the path for float32 inputs (true fp32
// contraction, needed for the 1e-5 bar) and for any shape the MFMA path does not cover.
//
// The accumulated score of the paper's Eq. 2 after the prompt, S_i = sum_{j>=i} a_i^j,
// is a column sum of the causal softmax matrix of Eq. 1.  The matrix is never stored:
//   pass 1 (rowstat): per query row j the running maximum and sum of exponentials over the
//                     keys i <= j, kept as  lse2_j = m_j + log2(l_j)  in the base-2 domain;
//   pass 2 (colsum):  per key tile, recompute the logits against every later query tile,
//                     p = 2^(t - lse2_j), and add the tile's column sums.  One workgroup
//                     owns a key tile, so its column sums stay in registers and are written
//                     once: no atomics on memory.
// Both passes work on 64x64 logit tiles, 4x4 per thread, with Q and K staged through LDS in
// slabs of 32 elements of the head dimension.
//
// History-window scores (Eq. 3 after the prompt: only the last w+1 query rows count) use the same
// two kernels with `window` = w >= 0: query tiles wholly before row len-1-w are skipped, and
// pass 2 also stores the window's attention rows, p = a_i^j at row j - j_first of a [w+1, cap]
// matrix per head, which the decode steps need to drop the row that leaves the window.
// window < 0 means no window.
#include "vatp_device.h"

namespace vatp {

namespace {

constexpr int kTile = 64;
constexpr int kSlab = 32;

template <typename T, int D>
__device__ __forceinline__ void load_slab_transposed(const T *__restrict__ base, int row0,
                                                     int n_rows, int x0, float (*dst)[kTile])
{
    // 256 threads: thread t loads row t/4, 8 consecutive elements at x0 + (t%4)*8.
    const int r = threadIdx.x >> 2;
    const int xs = (threadIdx.x & 3) * 8;
    float v[8];
    if (row0 + r < n_rows) {
        const T *src = base + static_cast<size_t>(row0 + r) * D + x0 + xs;
        if constexpr (sizeof(T) == 2) {
            Elt<bf16_t>::unpack(*reinterpret_cast<const uint4 *>(src), v);
        } else {
            Elt<float>::unpack(*reinterpret_cast<const uint4 *>(src), v);
            Elt<float>::unpack(*reinterpret_cast<const uint4 *>(src + 4), v + 4);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) dst[xs + e][r] = v[e];
}

// acc[a][c] = sum_x Q[qrow0 + ty*4 + a][x] * K[krow0 + tx*4 + c][x]
template <typename T, int D>
__device__ __forceinline__ void logit_tile(const T *__restrict__ Qu, const T *__restrict__ Ku,
                                           int qrow0, int krow0, int len, float (*Qs)[kTile],
                                           float (*Ks)[kTile], float acc[4][4])
{
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = 0.f;
    for (int x0 = 0; x0 < D; x0 += kSlab) {
        __syncthreads();
        load_slab_transposed<T, D>(Qu, qrow0, len, x0, Qs);
        load_slab_transposed<T, D>(Ku, krow0, len, x0, Ks);
        __syncthreads();
#pragma unroll 8
        for (int x = 0; x < kSlab; ++x) {
            const float4 qv = *reinterpret_cast<const float4 *>(&Qs[x][ty * 4]);
            const float4 kv = *reinterpret_cast<const float4 *>(&Ks[x][tx * 4]);
            const float qa[4] = {qv.x, qv.y, qv.z, qv.w};
            const float ka[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[a][c] = fmaf(qa[a], ka[c], acc[a][c]);
        }
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_rowstat_generic(const T *__restrict__ Q,
                                                               const T *__restrict__ K,
                                                               float *__restrict__ lse2,
                                                               BatchMeta meta, int n_heads,
                                                               int cap, float scale_log2, int window, int group)
{
    __shared__ __attribute__((aligned(16))) float Qs[kSlab][kTile];
    __shared__ __attribute__((aligned(16))) float Ks[kSlab][kTile];
    const int b = blockIdx.z, h = blockIdx.y;
    const int len = meta.len[b];
    const int j0 = blockIdx.x * kTile;
    if (j0 >= len) return;
    if (window >= 0 && j0 + kTile <= len - 1 - window) return;      // no query of this tile is in the window
    // h runs over the query heads; query head h reads the keys of K/V head h / group
    const size_t unit = static_cast<size_t>(b) * n_heads * group + h;
    const T *Qu = Q + unit * cap * D;
    const T *Ku = K + unit / group * cap * D;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;

    float m[4], l[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) { m[a] = -INFINITY; l[a] = 0.f; }

    for (int i0 = 0; i0 <= j0; i0 += kTile) {
        float acc[4][4];
        logit_tile<T, D>(Qu, Ku, j0, i0, len, Qs, Ks, acc);
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int j = j0 + ty * 4 + a;
            float t[4], tmax = -INFINITY;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int i = i0 + tx * 4 + c;
                t[c] = (i <= j && i < len) ? acc[a][c] * scale_log2 : -INFINITY;
                tmax = fmaxf(tmax, t[c]);
            }
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, off));
            // key 0 is visible to every query row, so after the first tile the maximum is finite
            const float m_new = fmaxf(m[a], tmax);
            float part = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) part += exp2f(t[c] - m_new);
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) part += __shfl_xor(part, off);
            l[a] = l[a] * exp2f(m[a] - m_new) + part;
            m[a] = m_new;
        }
    }
    if (tx == 0) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int j = j0 + ty * 4 + a;
            if (j < len) lse2[unit * cap + j] = m[a] + log2f(l[a]);
        }
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_colsum_generic(const T *__restrict__ Q,
                                                              const T *__restrict__ K,
                                                              const float *__restrict__ lse2,
                                                              float *__restrict__ S,
                                                              BatchMeta meta, int n_heads,
                                                              int cap, float scale_log2, int window,
                                                              float *__restrict__ hist, int group)
{
    __shared__ __attribute__((aligned(16))) float Qs[kSlab][kTile];
    __shared__ __attribute__((aligned(16))) float Ks[kSlab][kTile];
    __shared__ float red[16][kTile];
    const int b = blockIdx.z, h = blockIdx.y;
    const int len = meta.len[b];
    const int i0 = blockIdx.x * kTile;
    if (i0 >= len) return;
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const T *Ku = K + unit * cap * D;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;

    // first query row that counts, and the window's attention rows of this unit (w+1 of them, cap entries each)
    const int q_first = window >= 0 ? max(0, len - 1 - window) : 0;
    float *hu = hist ? hist + unit * static_cast<size_t>(window + 1) * cap : nullptr;
    float col[4] = {0.f, 0.f, 0.f, 0.f};
    const float inv_group = 1.f / static_cast<float>(group);      // (exactly 1 for one head)
    // the query heads that share this K/V head, one after the other (grouped-query attention; one otherwise):
    // their column sums add up in the same registers and the mean is taken at the end
    for (int qh = 0; qh < group; ++qh) {
        const T *Qu = Q + (unit * group + qh) * cap * D;
        const float *lu = lse2 + (unit * group + qh) * cap;
        for (int j0 = max(i0, q_first / kTile * kTile); j0 < len; j0 += kTile) {
            float acc[4][4];
            logit_tile<T, D>(Qu, Ku, j0, i0, len, Qs, Ks, acc);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int j = j0 + ty * 4 + a;
                if (j < len && j >= q_first) {
                    const float lj = lu[j];
                    float *hrow = hu ? hu + static_cast<size_t>(j - q_first) * cap : nullptr;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int i = i0 + tx * 4 + c;
                        if (i <= j) {
                            const float pr = exp2f(acc[a][c] * scale_log2 - lj);
                            col[c] += pr;
                            // (the group mean of the attention rows: this thread comes back to the same
                            // entry once per query head)
                            if (hrow) hrow[i] = qh == 0 ? pr * inv_group : hrow[i] + pr * inv_group;
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) red[ty][tx * 4 + c] = col[c];
    __syncthreads();
    if (threadIdx.x < kTile) {
        float s = 0.f;
#pragma unroll
        for (int y = 0; y < 16; ++y) s += red[y][threadIdx.x];
        const int i = i0 + threadIdx.x;
        if (i < len) S[unit * cap + i] = s * inv_group;
    }
}

// Row log-sum-exp handed in by an upstream attention kernel (natural logarithm) -> base 2.
__global__ __launch_bounds__(256) void lse_to_base2_kernel(const float *__restrict__ lse,
                                                           float *__restrict__ lse2, BatchMeta meta,
                                                           int n_heads, int cap)
{
    const int b = blockIdx.z, h = blockIdx.y;
    const int r = blockIdx.x * 256 + threadIdx.x;
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    if (r < meta.len[b]) lse2[unit * cap + r] = lse[unit * cap + r] * 1.44269504088896340736f;
}

}  // namespace

hipError_t launch_lse_to_base2(const float *lse, float *lse2, const BatchMeta &meta, const Geometry &g,
                               hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    const int q_heads = g.n_heads * g.group;           // one row log-sum-exp per query head
    hipLaunchKernelGGL(lse_to_base2_kernel, dim3((g.max_len + 255) / 256, q_heads, g.batch), dim3(256), 0, st, lse,
                       lse2, meta, q_heads, g.cap);
    return hipGetLastError();
}

hipError_t launch_prefill_generic(int dtype, int head_dim, const void *Q, const void *K,
                                  float *S, float *lse2, bool have_lse, int window, float *hist,
                                  const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    dim3 grid((g.max_len + kTile - 1) / kTile, g.n_heads, g.batch), block(256);
    dim3 grid_q(grid.x, g.n_heads * g.group, g.batch);        // row statistics: one pass per query head
#define VATP_PF(T, D)                                                                          \
    do {                                                                                       \
        if (!have_lse)                                                                         \
            hipLaunchKernelGGL((prefill_rowstat_generic<T, D>), grid_q, block, 0, st,          \
                               static_cast<const T *>(Q), static_cast<const T *>(K), lse2,     \
                               meta, g.n_heads, g.cap, g.scale_log2, window, g.group);         \
        hipLaunchKernelGGL((prefill_colsum_generic<T, D>), grid, block, 0, st,                 \
                           static_cast<const T *>(Q), static_cast<const T *>(K), lse2, S,      \
                           meta, g.n_heads, g.cap, g.scale_log2, window, hist, g.group);       \
    } while (0)
    if (dtype == VATP_F32 && head_dim == 64) VATP_PF(float, 64);
    else if (dtype == VATP_F32) VATP_PF(float, 128);
    else if (head_dim == 64) VATP_PF(bf16_t, 64);
    else VATP_PF(bf16_t, 128);             // (without a window this shape runs on the MFMA kernels instead)
#undef VATP_PF
    return hipGetLastError();
}

}  // namespace vatp
