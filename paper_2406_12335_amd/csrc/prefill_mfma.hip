// Prompt-pass scoring on the matrix cores (bf16 inputs, head_dim 128, gfx950).
//
// Accumulated attention score after the prompt (paper Eq. 2 with t = L-1):
//     S_i = sum_{j>=i} a_i^j ,   a^j = softmax over keys i<=j of c*<q_j,k_i>   (Eq. 1).
// The L x L matrix is never stored.  Two kernels, same skeleton:
//   rowstat  queries stationary, keys streamed:  per query j  lse2_j = log2 sum_i 2^(t_ji)
//   colsum   keys stationary, queries streamed:  S_i = sum_j 2^(t_ji - lse2_j)
// with t = c*log2(e)*<q,k>.
//
// Skeleton.  A workgroup of 4 wavefronts owns 256 "stationary" rows (64 per wavefront), kept
// for the whole kernel in registers as the B operand of v_mfma_f32_32x32x16_bf16 (columns of
// the logit tile).  The other matrix streams through LDS in stages of 64 rows (double
// buffered, one barrier per stage) and is the A operand (rows of the logit tile).  In the
// 32x32 accumulator a lane then holds ONE stationary column and 16 streamed rows, so the
// reduction each pass needs -- over keys for a query's row statistics, over queries for a
// key's column sum -- runs inside the lane; the two lane halves are merged once at the end
// with a single shuffle, and wavefronts own disjoint columns, so nothing is reduced through
// memory and there are no atomics.
//
// The contraction index (head dimension) may be permuted freely as long as both operands
// agree: lane half g takes the 16-byte chunk  s + 8g  of a row for MFMA step s.  LDS rows
// are 256 bytes; chunk c of row r is stored at chunk (c&8) | ((c&7) ^ ((r + 4*(c>>3)) & 7))
// so that the 16-byte reads of a 32x8-chunk operand fragment spread over all banks.
#include "vatp_device.h"

namespace vatp {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kD = 128;            // head_dim
constexpr int kStage = 64;         // streamed rows per LDS stage
constexpr int kWaveCols = 64;      // stationary rows per wavefront
constexpr int kBlockCols = 256;    // stationary rows per workgroup
constexpr int kChunksPerRow = kD * 2 / 16;   // 16-byte chunks per row = 16

__device__ __forceinline__ int swizzled_chunk(int row, int c) {
    return (c & 8) | ((c & 7) ^ ((row + ((c >> 3) << 2)) & 7));
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &u) { return __builtin_bit_cast(bf16x8, u); }

// Row offset inside a 32-row block of accumulator register v for lane half g.
__device__ __forceinline__ constexpr int acc_row(int v) { return 8 * (v / 4) + (v % 4); }

template <bool kColsum>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(const bf16_t *__restrict__ Q,
                                                              const bf16_t *__restrict__ K,
                                                              float *__restrict__ lse2,
                                                              float *__restrict__ S, BatchMeta meta,
                                                              int n_heads, int cap, int n_blocks,
                                                              float scale_log2)
{
    __shared__ uint4 stage[2][kStage * kChunksPerRow];     // 2 x 16 KiB
    __shared__ float lse_stage[2][kStage];

    const int b = blockIdx.z, h = blockIdx.y;
    const int len = meta.len[b];
    // heavier blocks first: rowstat work grows with the block index, colsum work shrinks
    const int blk = kColsum ? blockIdx.x : (n_blocks - 1 - blockIdx.x);
    const int base0 = blk * kBlockCols;
    if (base0 >= len) return;
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const uint4 *stat = reinterpret_cast<const uint4 *>((kColsum ? K : Q) + unit * cap * kD);
    const uint4 *strm = reinterpret_cast<const uint4 *>((kColsum ? Q : K) + unit * cap * kD);
    float *lse_u = lse2 + unit * cap;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, g = lane >> 5, n = lane & 31;
    const int w0 = base0 + wave * kWaveCols;           // first stationary row of this wavefront

    // stationary operand: 2 column blocks x 8 MFMA steps, 8 bf16 per lane each
    bf16x8 Bf[2][8];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int row = w0 + 32 * cb + n;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (row < len) raw = stat[static_cast<size_t>(row) * kChunksPerRow + s + 8 * g];
            Bf[cb][s] = as_bf16x8(raw);
        }
    }

    // stages of streamed rows this workgroup walks through
    const int t_begin = kColsum ? base0 / kStage : 0;
    const int last_row = kColsum ? len - 1 : min(base0 + kBlockCols - 1, len - 1);
    const int t_end = last_row / kStage;               // inclusive

    // thread's share of a stage: 4 chunks, rows tid/16 + 16 i, chunk tid%16
    const int ld_row = tid >> 4, ld_c = tid & 15;
    uint4 pre[4];
    float pre_lse = 0.f;
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = t * kStage + ld_row + 16 * i;
            pre[i] = (r < len) ? strm[static_cast<size_t>(r) * kChunksPerRow + ld_c] : make_uint4(0, 0, 0, 0);
        }
        if (kColsum && tid < kStage) {
            const int r = t * kStage + tid;
            pre_lse = (r < len) ? lse_u[r] : INFINITY;   // 2^(t - inf) = 0: rows past the end add nothing
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = ld_row + 16 * i;
            stage[buf][r * kChunksPerRow + swizzled_chunk(r, ld_c)] = pre[i];
        }
        if (kColsum && tid < kStage) lse_stage[buf][tid] = pre_lse;
    };

    // running state, per column block
    float m_run[2] = {-1e30f, -1e30f}, l_run[2] = {0.f, 0.f};   // rowstat
    float col[2] = {0.f, 0.f};                                  // colsum

    fetch(t_begin);
    commit(0);
    __syncthreads();

    for (int t = t_begin; t <= t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        if (t < t_end) fetch(t + 1);

        const int s0 = t * kStage;                      // first streamed row of the stage
        // rowstat: streamed = keys, stationary = queries; a key may attend iff key <= query
        // colsum : streamed = queries, stationary = keys
        const bool skip = kColsum ? (s0 + kStage - 1 < w0) : (s0 > w0 + kWaveCols - 1);
        if (!skip) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int r0 = s0 + 32 * kb;            // first streamed row of this row block
                bf16x8 Af[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const int r = 32 * kb + n;
                    Af[s] = as_bf16x8(stage[buf][r * kChunksPerRow + swizzled_chunk(r, s + 8 * g)]);
                }
                float lse_v[16];
                if (kColsum) {
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const float4 x = *reinterpret_cast<const float4 *>(&lse_stage[buf][32 * kb + 8 * q4 + 4 * g]);
                        lse_v[4 * q4 + 0] = x.x; lse_v[4 * q4 + 1] = x.y; lse_v[4 * q4 + 2] = x.z; lse_v[4 * q4 + 3] = x.w;
                    }
                }
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const int c0 = w0 + 32 * cb;        // first stationary row of this column block
                    // whole 32x32 tile above the diagonal?
                    const bool dead = kColsum ? (r0 + 31 < c0) : (r0 > c0 + 31);
                    if (dead) continue;
                    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 8; ++s)
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Af[s], Bf[cb][s], acc, 0, 0, 0);
                    // does the diagonal cross this tile?
                    const bool diag = kColsum ? (r0 < c0 + 31) : (r0 + 31 > c0);
                    // lane's stationary index minus the first streamed row it holds
                    const int d0 = (c0 + n) - (r0 + 4 * g);
                    if (!kColsum) {
                        if (diag) {
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[v] = (acc_row(v) <= d0) ? acc[v] : -INFINITY;
                        }
                        float tmax = acc[0];
#pragma unroll
                        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[v]);
                        const float m_new = fmaxf(m_run[cb], tmax * scale_log2);
                        float part0 = 0.f, part1 = 0.f;
#pragma unroll
                        for (int v = 0; v < 16; v += 2) {
                            part0 += __builtin_amdgcn_exp2f(fmaf(acc[v], scale_log2, -m_new));
                            part1 += __builtin_amdgcn_exp2f(fmaf(acc[v + 1], scale_log2, -m_new));
                        }
                        l_run[cb] = l_run[cb] * __builtin_amdgcn_exp2f(m_run[cb] - m_new) + (part0 + part1);
                        m_run[cb] = m_new;
                    } else {
                        float part0 = 0.f, part1 = 0.f;
                        if (diag) {
#pragma unroll
                            for (int v = 0; v < 16; v += 2) {
                                const float p0 = __builtin_amdgcn_exp2f(fmaf(acc[v], scale_log2, -lse_v[v]));
                                const float p1 = __builtin_amdgcn_exp2f(fmaf(acc[v + 1], scale_log2, -lse_v[v + 1]));
                                part0 += (acc_row(v) >= d0) ? p0 : 0.f;
                                part1 += (acc_row(v + 1) >= d0) ? p1 : 0.f;
                            }
                        } else {
#pragma unroll
                            for (int v = 0; v < 16; v += 2) {
                                part0 += __builtin_amdgcn_exp2f(fmaf(acc[v], scale_log2, -lse_v[v]));
                                part1 += __builtin_amdgcn_exp2f(fmaf(acc[v + 1], scale_log2, -lse_v[v + 1]));
                            }
                        }
                        col[cb] += part0 + part1;
                    }
                }
            }
        }

        if (t < t_end) commit(buf ^ 1);
        __syncthreads();
    }

    // merge the two lane halves (same stationary column, complementary streamed rows)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int idx = w0 + 32 * cb + n;
        if (!kColsum) {
            const float m_o = __shfl_xor(m_run[cb], 32), l_o = __shfl_xor(l_run[cb], 32);
            const float m = fmaxf(m_run[cb], m_o);
            const float l = l_run[cb] * __builtin_amdgcn_exp2f(m_run[cb] - m) + l_o * __builtin_amdgcn_exp2f(m_o - m);
            if (g == 0 && idx < len) lse_u[idx] = m + __log2f(l);
        } else {
            const float s = col[cb] + __shfl_xor(col[cb], 32);
            if (g == 0 && idx < len) S[unit * cap + idx] = s;
        }
    }
}

}  // namespace

hipError_t launch_prefill_mfma(const void *Q, const void *K, float *S, float *lse2,
                               const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    const int n_blocks = (g.max_len + kBlockCols - 1) / kBlockCols;
    dim3 grid(n_blocks, g.n_heads, g.batch), block(256);
    hipLaunchKernelGGL((prefill_mfma_kernel<false>), grid, block, 0, st, static_cast<const bf16_t *>(Q),
                       static_cast<const bf16_t *>(K), lse2, S, meta, g.n_heads, g.cap, n_blocks, g.scale_log2);
    hipLaunchKernelGGL((prefill_mfma_kernel<true>), grid, block, 0, st, static_cast<const bf16_t *>(Q),
                       static_cast<const bf16_t *>(K), lse2, S, meta, g.n_heads, g.cap, n_blocks, g.scale_log2);
    return hipGetLastError();
}

}  // namespace vatp
