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
// in registers as the B operand of v_mfma_f32_32x32x16_bf16 (columns of the logit tile).  The
// other matrix streams through LDS in stages of 64 rows (double buffered, one barrier per
// stage) and is the A operand (rows of the logit tile).  In the 32x32 accumulator a lane then
// holds ONE stationary column and 16 streamed rows, so the reduction each pass needs -- over
// keys for a query's row statistics, over queries for a key's column sum -- runs inside the
// lane; the two lane halves are merged once at the end with a single shuffle, and wavefronts
// own disjoint columns, so nothing is reduced through memory and there are no atomics.
//
// The exponentials cost more vector-ALU time than the contraction costs matrix time, so the
// two are overlapped inside every wavefront: while the 16 MFMAs of one pair of tiles (32
// streamed rows x 64 columns) execute, the lane works through the exponentials of the
// previous pair ("pending" accumulators).  Causal masking is applied to a finished
// accumulator by writing -inf into the masked entries, which both epilogues turn into 0.
//
// Causal work per 256-row block grows (rowstat) or shrinks (colsum) linearly with the block
// index; a workgroup therefore takes the pair of blocks (x, n_blocks-1-x), which gives every
// workgroup the same amount of work.
//
// The contraction index (head dimension) may be permuted freely as long as both operands
// agree: lane half g takes the 16-byte chunk  s + 8g  of a row for MFMA step s.  LDS rows
// are 256 bytes; chunk c of row r is stored at chunk  c ^ (r & 15).
#include <type_traits>

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

__device__ __forceinline__ int swizzled_chunk(int row, int c) { return c ^ (row & 15); }

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &u) { return __builtin_bit_cast(bf16x8, u); }

// Row offset inside a 32-row block of accumulator register v (lane half g adds 4g).
__device__ __forceinline__ constexpr int acc_row(int v) { return 8 * (v / 4) + (v % 4); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Scheduling request for two MFMA slots: one MFMA, V0 vector-ALU instructions, one MFMA, V1
// vector-ALU instructions, and optionally one LDS read (0x008 MFMA, 0x002 VALU, 0x100 DS read).
template <int V0, int V1, bool kRead>
__device__ __forceinline__ void sched_two_slots()
{
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, V0, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, V1, 0);
    if constexpr (kRead) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
}

template <bool kColsum>
struct Pending {               // a finished pair of 32x32 tiles awaiting its exponentials
    floatx16 acc[2];
    float lse[kColsum ? 16 : 1];
};

template <bool kColsum>
struct Running {                 // per column block: rowstat (m, l) or colsum partial sum
    float m[2], l[2], col[2];
};

// The exponentials of a pending pair, cut into 16 pieces so that one piece can follow each
// MFMA of the next pair.  piece < 0 runs everything that is left after piece 15.
template <bool kColsum>
struct Epilogue {
    float ref[2], corr[2], part[2], tmax[2];

    __device__ __forceinline__ void piece(int i, const Pending<kColsum> &p, const Running<kColsum> &run,
                                          float scale)
    {
        if constexpr (kColsum) {
            if (i == 0) { part[0] = 0.f; part[1] = 0.f; }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) part[cb] += fast_exp2(fmaf(p.acc[cb][i], scale, -p.lse[i]));
        } else {
            if (i < 2) {                                   // tile maximum of column block i
                float t = fmaxf(p.acc[i][0], p.acc[i][1]);
#pragma unroll
                for (int v = 2; v < 16; v += 2) t = fmaxf(t, fmaxf(p.acc[i][v], p.acc[i][v + 1]));
                tmax[i] = t;
            } else if (i == 2) {
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    ref[cb] = fmaxf(run.m[cb], tmax[cb] * scale);
                    corr[cb] = fast_exp2(run.m[cb] - ref[cb]);
                    part[cb] = 0.f;
                }
            } else {
                const int v = i - 3;
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) part[cb] += fast_exp2(fmaf(p.acc[cb][v], scale, -ref[cb]));
            }
        }
    }

    __device__ __forceinline__ void finish(const Pending<kColsum> &p, Running<kColsum> &run, float scale)
    {
        if constexpr (kColsum) {
            run.col[0] += part[0];
            run.col[1] += part[1];
        } else {
#pragma unroll
            for (int v = 13; v < 16; ++v)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) part[cb] += fast_exp2(fmaf(p.acc[cb][v], scale, -ref[cb]));
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                run.l[cb] = run.l[cb] * corr[cb] + part[cb];
                run.m[cb] = ref[cb];
            }
        }
    }
};

template <bool kColsum>
__global__ __launch_bounds__(256) void prefill_mfma_kernel(const bf16_t *__restrict__ Q,
                                                           const bf16_t *__restrict__ K,
                                                           float *__restrict__ lse2,
                                                           float *__restrict__ S, BatchMeta meta,
                                                           int n_heads, int cap, int n_blocks,
                                                           float scale_log2)
{
    __shared__ uint4 stage[2][kStage * kChunksPerRow];     // 2 x 16 KiB
    __shared__ __attribute__((aligned(16))) float lse_stage[2][kStage];

    const int b = blockIdx.z, h = blockIdx.y;
    const int len = meta.len[b];
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const uint4 *stat = reinterpret_cast<const uint4 *>((kColsum ? K : Q) + unit * cap * kD);
    const uint4 *strm = reinterpret_cast<const uint4 *>((kColsum ? Q : K) + unit * cap * kD);
    float *lse_u = lse2 + unit * cap;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, g = lane >> 5, n = lane & 31;
    const int ld_row = tid >> 4, ld_c = tid & 15;      // this thread's share of a stage

    for (int job = 0; job < 2; ++job) {
        const int blk = job == 0 ? static_cast<int>(blockIdx.x) : n_blocks - 1 - static_cast<int>(blockIdx.x);
        if (job == 1 && blk == static_cast<int>(blockIdx.x)) break;      // odd count: the middle block once
        const int base0 = blk * kBlockCols;
        if (base0 >= len) continue;
        const int w0 = base0 + wave * kWaveCols;       // first stationary row of this wavefront

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

        Running<kColsum> run;
        run.m[0] = run.m[1] = -1e30f;
        run.l[0] = run.l[1] = 0.f;
        run.col[0] = run.col[1] = 0.f;
        // a neutral pending pair: -inf logits turn into zeros in both epilogues
        Pending<kColsum> pend;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            pend.acc[0][v] = -INFINITY;
            pend.acc[1][v] = -INFINITY;
            if (kColsum) pend.lse[v] = 0.f;
        }

        fetch(t_begin);
        commit(0);
        __syncthreads();

        for (int t = t_begin; t <= t_end; ++t) {
            const int buf = (t - t_begin) & 1;
            if (t < t_end) fetch(t + 1);

            const int s0 = t * kStage;                      // first streamed row of the stage
            // rowstat: streamed = keys, stationary = queries; a key counts iff key <= query
            // colsum : streamed = queries, stationary = keys
            const bool skip = kColsum ? (s0 < w0) : (s0 > w0);
            if (!skip) {
                // One stage = two pairs of tiles.  The body is branch-free (the diagonal variant is
                // a separate instantiation) so that MFMAs and exponentials share one basic block.
                auto do_stage = [&](auto diag_tag) {
                    constexpr bool kDiag = decltype(diag_tag)::value;
                    // the two instantiations must not share a hoisted prefix: the pending pair's
                    // exponentials belong next to this stage's MFMAs
                    // (the scale is re-read through an opaque asm so nothing that uses it can move up)
                    float scale = scale_log2;
                    asm volatile("; stage variant %1" : "+s"(scale) : "n"(kDiag ? 1 : 0));
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        const int ar = 32 * kb + n;            // this lane's row of the streamed tile
                        Pending<kColsum> next;
                        if (kColsum) {
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) {
                                const float4 x =
                                    *reinterpret_cast<const float4 *>(&lse_stage[buf][32 * kb + 8 * q4 + 4 * g]);
                                next.lse[4 * q4 + 0] = x.x; next.lse[4 * q4 + 1] = x.y;
                                next.lse[4 * q4 + 2] = x.z; next.lse[4 * q4 + 3] = x.w;
                            }
                        }
#pragma unroll
                        for (int v = 0; v < 16; ++v) { next.acc[0][v] = 0.f; next.acc[1][v] = 0.f; }
                        Epilogue<kColsum> epi;
                        bf16x8 a[8];
#pragma unroll
                        for (int s = 0; s < 8; ++s)
                            a[s] = as_bf16x8(stage[buf][ar * kChunksPerRow + swizzled_chunk(ar, s + 8 * g)]);
#pragma unroll
                        for (int s = 0; s < 8; ++s) {
                            next.acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], Bf[0][s], next.acc[0], 0, 0, 0);
                            epi.piece(2 * s, pend, run, scale);
                            next.acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], Bf[1][s], next.acc[1], 0, 0, 0);
                            epi.piece(2 * s + 1, pend, run, scale);
                        }
                        epi.finish(pend, run, scale);
                        // keep the pending pair's results inside this block (no sinking past it)
                        if constexpr (kColsum) asm volatile("" : "+v"(run.col[0]), "+v"(run.col[1]));
                        else asm volatile("" : "+v"(run.l[0]), "+v"(run.l[1]), "+v"(run.m[0]), "+v"(run.m[1]));
                        // Issue order asked of the scheduler: all LDS reads of the pair first, then a
                        // run of the pending pair's vector work to cover their latency, then one
                        // MFMA per slice of exponentials.
                        __builtin_amdgcn_sched_group_barrier(0x100, kColsum ? 12 : 8, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
                        sched_two_slots<5, 5, false>(); sched_two_slots<5, 5, false>(); sched_two_slots<5, 5, false>();
                        sched_two_slots<5, 5, false>(); sched_two_slots<5, 5, false>(); sched_two_slots<5, 5, false>();
                        sched_two_slots<5, 5, false>(); sched_two_slots<5, 5, false>();
                        if constexpr (kDiag) {
                            // mask the entries above the diagonal of the finished pair
#pragma unroll
                            for (int cb = 0; cb < 2; ++cb) {
                                // lane's stationary index minus the first streamed row it holds
                                const int d0 = (w0 + 32 * cb + n) - (s0 + 32 * kb + 4 * g);
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const bool ok = kColsum ? (acc_row(v) >= d0) : (acc_row(v) <= d0);
                                    next.acc[cb][v] = ok ? next.acc[cb][v] : -INFINITY;
                                }
                            }
                        }
                        pend = next;
                    }
                };
                if (s0 == w0) do_stage(std::true_type{});
                else do_stage(std::false_type{});
            }

            if (t < t_end) commit(buf ^ 1);
            __syncthreads();
        }

        // the last pair still waits for its exponentials
        {
            Epilogue<kColsum> epi;
#pragma unroll
            for (int i = 0; i < 16; ++i) epi.piece(i, pend, run, scale_log2);
            epi.finish(pend, run, scale_log2);
        }

        // merge the two lane halves (same stationary column, complementary streamed rows)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int idx = w0 + 32 * cb + n;
            if (!kColsum) {
                const float m_o = __shfl_xor(run.m[cb], 32), l_o = __shfl_xor(run.l[cb], 32);
                const float m = fmaxf(run.m[cb], m_o);
                const float l = run.l[cb] * fast_exp2(run.m[cb] - m) + l_o * fast_exp2(m_o - m);
                if (g == 0 && idx < len) lse_u[idx] = m + __log2f(l);
            } else {
                const float s = run.col[cb] + __shfl_xor(run.col[cb], 32);
                if (g == 0 && idx < len) S[unit * cap + idx] = s;
            }
        }
    }
}

}  // namespace

hipError_t launch_prefill_mfma(const void *Q, const void *K, float *S, float *lse2,
                               const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    const int n_blocks = (g.max_len + kBlockCols - 1) / kBlockCols;
    dim3 grid((n_blocks + 1) / 2, g.n_heads, g.batch), block(256);
    hipLaunchKernelGGL((prefill_mfma_kernel<false>), grid, block, 0, st, static_cast<const bf16_t *>(Q),
                       static_cast<const bf16_t *>(K), lse2, S, meta, g.n_heads, g.cap, n_blocks, g.scale_log2);
    hipLaunchKernelGGL((prefill_mfma_kernel<true>), grid, block, 0, st, static_cast<const bf16_t *>(Q),
                       static_cast<const bf16_t *>(K), lse2, S, meta, g.n_heads, g.cap, n_blocks, g.scale_log2);
    return hipGetLastError();
}

}  // namespace vatp
