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
// other matrix streams through LDS in stages of 64 rows and is the A operand (rows of the
// logit tile).  In the 32x32 accumulator a lane then holds ONE stationary column and 16
// streamed rows, so the reduction each pass needs -- over keys for a query's row statistics,
// over queries for a key's column sum -- runs inside the lane; the two lane halves are merged
// once at the end with a single shuffle, and wavefronts own disjoint columns, so nothing is
// reduced through memory and there are no atomics.
//
// Streaming.  Stages are copied global -> LDS by the load unit itself
// (global_load_lds_dwordx4: each lane's 16 bytes land at LDS base + 16*lane, no registers),
// three stages ahead of the one being consumed, into a ring of four 16 KiB buffers; one
// s_barrier per stage.  The copies are issued from inline assembly, so their completion is
// tracked by hand: a wavefront waits until at most the copies of the younger stages are
// outstanding (s_waitcnt vmcnt) before the barrier that publishes a stage.  LDS rows are 256
// bytes; chunk c of row r sits at chunk c ^ (r & 15), which the copy realises on the source
// side (the lane that fills LDS chunk p of row r fetches global chunk p ^ (r & 15)).
//
// The exponentials cost more vector-ALU time than the contraction costs matrix time, so the
// two are overlapped inside every wavefront: while the 16 MFMAs of one pair of tiles (32
// streamed rows x 64 columns) execute, the lane works through the exponentials of the
// previous pair ("pending" accumulators).  Masking (causal diagonal, rows past the end) is
// applied to a finished accumulator by writing -inf into the masked entries, which both
// epilogues turn into 0.
//
// Causal work per 256-row block grows (rowstat) or shrinks (colsum) linearly with the block
// index; a workgroup therefore takes the pair of blocks (x, n_blocks-1-x), which gives every
// workgroup the same amount of work.
//
// History-window scores (Eq. 3 after the prompt: only the last w+1 query rows count) reuse both
// kernels (kWindow).  The row-statistics pass then has only the window's few query blocks to
// work on, so the keys they stream are cut into ranges, one workgroup per (block, range), each
// leaving a partial log-sum-exp that a small kernel merges.  The column-sum pass starts
// streaming at the window's first query, masks the rows before it, and also stores the
// window's attention rows (row j - j_first of a [w+1, cap] matrix per head) through a buffer
// descriptor whose bounds check drops the rows outside the window by itself.
//
// Grouped queries (g query heads per K/V head; paper, Limitations section): the token score is the mean over
// the group of the heads' column sums.  Row statistics are per query head (one unit per query head, streaming
// its K/V head's keys).  The column-sum pass keeps one unit per K/V head (kGrouped): a job streams the queries
// of the group's heads one after the other into the same accumulators, so K is loaded once per group; on a
// small grid the heads are dealt out to several workgroups whose partial sums a small kernel adds.  With a
// history window the heads go innermost instead (every 64-row stage of queries once per head): a lane then
// meets the same (query, key) entries of all heads in turn, adds their weights in registers and stores the
// stage's attention rows, already averaged, once.
//
// The contraction index (head dimension) may be permuted freely as long as both operands
// agree: lane half g takes the 16-byte chunk  s + 8g  of a row for MFMA step s.
#include <type_traits>

#include "vatp_device.h"

namespace vatp {

namespace {

typedef __attribute__((address_space(3))) char lds_char;

constexpr int kD = 128;            // head_dim
constexpr int kStage = 64;         // streamed rows per LDS stage
constexpr int kRing = 4;           // LDS stage buffers
constexpr unsigned kComputeUnits = 256;
constexpr int kAhead = kRing - 1;  // stages in flight beyond the one being consumed
constexpr int kWaveCols = 64;      // stationary rows per wavefront
constexpr int kBlockCols = 256;    // stationary rows per workgroup
constexpr int kChunksPerRow = kD * 2 / 16;   // 16-byte chunks per row = 16
constexpr int kStageBytes = kStage * kD * 2; // 16 KiB
#ifndef VATP_LEAD_VALU
#define VATP_LEAD_VALU 12
#endif
#ifndef VATP_SLOT_VALU
#define VATP_SLOT_VALU 5
#endif
constexpr int kLeadValu = VATP_LEAD_VALU;    // vector instructions asked for between the LDS reads and the first MFMA
constexpr int kSlotValu = VATP_SLOT_VALU;    // vector instructions asked for after every MFMA

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Scheduling request for two MFMA slots: one MFMA, V0 vector-ALU instructions, one MFMA, V1
// vector-ALU instructions (0x008 MFMA, 0x002 VALU).
template <int V0, int V1>
__device__ __forceinline__ void sched_two_slots()
{
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, V0, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, V1, 0);
}

// Wait until at most kPending of this wavefront's vector-memory operations are outstanding,
// then meet the other wavefronts.  The "memory" clobber keeps LDS reads below it.
template <int kPending>
__device__ __forceinline__ void wait_copies_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kPending) : "memory");
}

template <bool kColsum>
struct Pending {                 // a finished pair of 32x32 tiles awaiting its exponentials
    floatx16 acc[2];
    float lse[kColsum ? 16 : 1];
    unsigned hist_off[2];        // windowed column sums: byte offset of (first row held, column) per column block
};

// Arguments of the history-window variant (unused otherwise).
struct WindowPass {
    int window;                  // w
    float *hist;                 // [units, w + 1, cap] attention rows of the window, may be NULL
    float *lse_part;             // [n_splits, units, cap] partial row statistics
    int n_splits, split_stages;  // key ranges per query block, 64-row stages per range
    int n_qb;                    // query blocks per head that can touch the window
};

template <bool kColsum>
struct Running {                 // per column block: rowstat (m, l) or colsum partial sum
    float m[2], l[2], col[2];
};

// The exponentials of a pending pair, cut into 16 pieces so that one piece can follow each
// MFMA of the next pair; finish() runs what is left after piece 15.
template <bool kColsum>
struct Epilogue {
    float ref[2], corr[2], part[2], tmax[2];

    // kStore: 0 nothing, 1 the attention weights are stored through hist_rsrc, 2 they are added to the sums
    // `group_sum` that a lane keeps for the query heads of a group (the stage's rows are stored once, after the
    // last head)
    template <int kStore = 0>
    __device__ __forceinline__ void piece(int i, const Pending<kColsum> &p, const Running<kColsum> &run,
                                          float scale, __amdgpu_buffer_rsrc_t hist_rsrc, int row_bytes,
                                          float (*group_sum)[16] = nullptr)
    {
        if constexpr (kColsum) {
            if (i == 0) { part[0] = 0.f; part[1] = 0.f; }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const float pr = fast_exp2(fmaf(p.acc[cb][i], scale, -p.lse[i]));
                part[cb] += pr;
                // offsets outside the descriptor (rows before or after the window, columns past the
                // sequence) are dropped by the store unit
                if constexpr (kStore == 1)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_int(pr), hist_rsrc,
                                                          p.hist_off[cb] + acc_row(i) * row_bytes, 0, 0);
                else if constexpr (kStore == 2)
                    group_sum[cb][i] += pr;
            }
        } else {
            if (i < 2) {                                   // tile maximum of column block i
                // a linear chain, so that every two steps fuse into one three-operand maximum
                float t = p.acc[i][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) t = fmaxf(t, p.acc[i][v]);
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

// Norms of 64 consecutive value rows by one wavefront.  Same arithmetic as l1norm_kernel: 16 lanes per
// row, 8 elements each in order, then an all-reduce over the row's 16 lanes; all 16 loads of a lane are
// issued before the first is used.
template <int kNorm>
__device__ __forceinline__ void value_norms_64(const uint4 *__restrict__ Vu, float *__restrict__ nu, int row0, int len,
                                               int lane)
{
    const int sub = lane & 15, rr = lane >> 4;
    uint4 raw[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const int row = row0 + 4 * p + rr;
        raw[p] = row < len ? Vu[static_cast<size_t>(row) * kChunksPerRow + sub] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const int row = row0 + 4 * p + rr;
        const float value = row_norm<bf16_t, 16>(kNorm, raw[p]);
        if (sub == 0 && row < len) nu[row] = value;
    }
}

template <bool kColsum, int kHalves, bool kWindow = false, bool kGrouped = false>
__global__ __launch_bounds__(256 * kHalves) void prefill_mfma_kernel(const bf16_t *__restrict__ Q,
                                                           const bf16_t *__restrict__ K,
                                                           float *__restrict__ lse2,
                                                           float *__restrict__ S, BatchMeta meta,
                                                           int n_heads, int n_units, int cap,
                                                           int n_blocks, float scale_log2, WindowPass win,
                                                           const bf16_t *__restrict__ V, float *__restrict__ nrm,
                                                           int norm, int group, int splits)
{
    static_assert(!kWindow || kHalves == 1, "the windowed passes use 4-wavefront workgroups");
    static_assert(!kGrouped || kColsum, "only the column-sum passes loop over a group's query heads");
    constexpr bool kSplitKeys = kWindow && !kColsum;      // windowed row statistics: one (block, key range) per workgroup
    // A ring slot holds kHalves sub-stages of 64 streamed rows; wavefront w works on sub-stage
    // w / 4 of every slot for the 64 stationary rows of column group w % 4.  With kHalves = 2
    // a workgroup has two wavefronts per SIMD (used when the grid has too few workgroups for
    // two of them to share a compute unit).
    constexpr int kSlotRows = kStage * kHalves;
    constexpr int kSlotBytes = kStageBytes * kHalves;
    __shared__ uint4 stage[kRing][kSlotRows * kChunksPerRow];   // filled by the load unit
    __shared__ __attribute__((aligned(16))) float lse_stage[kRing][kSlotRows];
    __shared__ float merge_buf[kHalves == 2 ? 2 : 1][kBlockCols];

    // Workgroups are handed to the 8 XCDs round-robin by linear id.  All block pairs of one
    // (batch, head) unit are given ids that are equal mod 8, so the unit's streamed matrix is
    // pulled into one XCD's L2 once instead of into all eight.
    const int n_pairs = kSplitKeys ? win.n_qb * win.n_splits : (n_blocks + 1) / 2;
    const int xcd = blockIdx.x & 7, in_xcd = blockIdx.x >> 3;
    const int slot_i = xcd + 8 * (in_xcd / n_pairs);
    const int pair = in_xcd % n_pairs;
    if (slot_i >= n_units) return;
    // (grouped column sums on a small grid: `splits` workgroups share a K/V head, each taking group / splits
    // of its query heads and leaving a partial column sum; n_units then counts K/V heads x splits)
    const int unit_i = kGrouped ? __builtin_amdgcn_readfirstlane(slot_i / splits) : slot_i;
    const int split = kGrouped ? slot_i - unit_i * splits : 0;
    const int b = unit_i / n_heads;
    const int len = meta.len[b];
    const int q_first = kWindow ? max(0, len - 1 - win.window) : 0;     // first query row that counts
    const size_t unit = static_cast<size_t>(unit_i);
    // Grouped-query attention (group > 1; paper, Limitations section): query head u belongs to K/V head
    // u / group.  The row-statistics pass has one unit per query head (n_heads then counts query heads) and
    // streams the keys of that head's K/V head; the column-sum pass (kGrouped) has one unit per K/V head
    // and streams the queries of its `group` query heads one after the other into the same column sums.
    const uint4 *stat = reinterpret_cast<const uint4 *>((kColsum ? K : Q) + unit * cap * kD);
    const bf16_t *const strm0 = kColsum ? Q + unit * group * cap * kD : K + unit / group * cap * kD;
    float *const lse_u0 = lse2 + (kColsum ? unit * group : unit) * cap;
    const bf16_t *strm = strm0;
    float *lse_u = lse_u0;
    // windowed column sums: descriptor over this head's [w + 1, cap] matrix of attention rows
    // (no matrix, or another kind of pass: zero records, every store is dropped)
    const bool with_hist = kWindow && kColsum && win.hist != nullptr;
    const __amdgpu_buffer_rsrc_t hist_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        with_hist ? win.hist + unit * static_cast<size_t>(win.window + 1) * cap : nullptr, 0,
        with_hist ? (win.window + 1) * cap * 4 : 0, 0x00020000);

    const float inv_group = 1.f / static_cast<float>(group);     // the group mean (exactly 1 for one head)
    const float log2_group = log2f(static_cast<float>(group));
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = wave & 3, half = wave >> 2;      // column group, sub-stage
    const int lane = tid & 63, g = lane >> 5, n = lane & 31;

    const unsigned lds_stage0 = static_cast<unsigned>(reinterpret_cast<size_t>((lds_char *)(char *)&stage[0][0]));
    const unsigned lds_lse0 = static_cast<unsigned>(reinterpret_cast<size_t>((lds_char *)(char *)&lse_stage[0][0]));

    // Copy stage t (kSlotRows streamed rows) into ring slot `slot`.  This wavefront moves rows
    // 16*wave .. 16*wave+15, four rows (1 KiB) per instruction.  Rows past the end of the
    // sequence are redirected to its last row (any finite data: they are masked later).
    auto copy_stage = [&](int t, int slot) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 16 * wave + 4 * i + (lane >> 4);           // row inside the stage
            const int c = (lane & 15) ^ (r & 15);                    // global chunk for LDS chunk lane&15
            const int grow = min(t * kSlotRows + r, len - 1);
            const unsigned voff = static_cast<unsigned>(grow) * (kD * 2) + c * 16;
            const unsigned m0v = lds_stage0 + slot * kSlotBytes + (16 * wave + 4 * i) * (kD * 2);
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0v), "v"(voff), "s"(strm)
                         : "memory");
        }
        if (kColsum && cw == 0) {
            const int grow = min(t * kSlotRows + kStage * half + lane, len - 1);
            const unsigned voff = static_cast<unsigned>(grow) * 4;
            const unsigned m0v = lds_lse0 + (slot * kSlotRows + kStage * half) * 4;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" ::"s"(m0v), "v"(voff), "s"(lse_u)
                         : "memory");
        }
    };
    // copies per stage issued by this wavefront (column group 0 also brings the lse values)
    const bool extra_copy = kColsum && cw == 0;
    // A job is one block of stationary rows; with grouped queries it is walked once per query head
    // (`run` and the stationary operand live on from one head to the next).
    // (Windowed column sums of a group, kBand, go through the heads inside the stage loop instead: see there.)
    constexpr bool kBand = kWindow && kColsum && kGrouped;
    const int n_qh = (kGrouped && !kBand) ? __builtin_amdgcn_readfirstlane(group / splits) : 1;
    bf16x8 Bf[2][8] = {};
    Running<kColsum> run;
    for (int it = 0, n_it = (kSplitKeys ? 1 : 2) * n_qh; it < n_it; ++it) {
        const int job = kGrouped ? (it >= n_qh ? 1 : 0) : it, qh = kGrouped ? it - job * n_qh : 0;     // (at most two jobs)
        int blk = job == 0 ? pair : n_blocks - 1 - pair;
        if constexpr (kSplitKeys) blk = q_first / kBlockCols + pair / win.n_splits;
        if (!kSplitKeys && job == 1 && blk == pair) break;   // odd count: the middle block once
        const int base0 = blk * kBlockCols;
        if (base0 >= len) continue;
        const int w0 = base0 + cw * kWaveCols;         // first stationary row of this wavefront

        // stages of streamed rows this workgroup walks through
        int t_begin = kColsum ? max(base0, q_first) / kSlotRows : 0;
        const int last_row = kColsum ? len - 1 : min(base0 + kBlockCols - 1, len - 1);
        int t_end = last_row / kSlotRows;                  // inclusive
        if constexpr (kSplitKeys) {                        // this workgroup's range of keys
            t_begin = (pair % win.n_splits) * win.split_stages;
            t_end = min(t_end, t_begin + win.split_stages - 1);
            if (t_begin > t_end) continue;
        }

        if constexpr (kGrouped && !kBand) {
            strm = strm0 + static_cast<size_t>(split * n_qh + qh) * cap * kD;
            lse_u = lse_u0 + static_cast<size_t>(split * n_qh + qh) * cap;
        }
        // kBand: the ring holds "virtual" stages v = (stage t, query head h), h innermost, so that a lane meets
        // the same (query row, key) entries of all heads of the group one after the other and can add them up
        // in registers.  The copy front runs kAhead virtual stages ahead.
        const int n_virtual = kBand ? (t_end - t_begin + 1) * group : 0;
        int issued = 0, copy_t = t_begin, copy_h = 0, cur_v = 0;
        auto issue_copy = [&]() __attribute__((always_inline)) {
            strm = strm0 + static_cast<size_t>(copy_h) * cap * kD;
            lse_u = lse_u0 + static_cast<size_t>(copy_h) * cap;
            copy_stage(copy_t, issued & (kRing - 1));
            ++issued;
            if (++copy_h == group) { copy_h = 0; ++copy_t; }
        };
        if constexpr (kBand) {
#pragma unroll
            for (int k = 0; k < kAhead; ++k)
                if (issued < n_virtual) issue_copy();
        } else {
#pragma unroll
            for (int k = 0; k < kAhead; ++k)
                if (t_begin + k <= t_end) copy_stage(t_begin + k, k);
        }

        // The column-sum pass visits every block of keys once: it also leaves the norm of the value rows
        // of its block (paper Eq. 4), 64 rows per wavefront, while the first stages are on their way.
        if constexpr (kColsum) {
            if (V != nullptr && half == 0 && qh == 0 && split == 0) {
                const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * kD);
                float *nu = nrm + unit * cap;
                switch (norm) {
                case VATP_NORM_L1: value_norms_64<VATP_NORM_L1>(Vu, nu, w0, len, lane); break;
                case VATP_NORM_L2: value_norms_64<VATP_NORM_L2>(Vu, nu, w0, len, lane); break;
                case VATP_NORM_LINF: value_norms_64<VATP_NORM_LINF>(Vu, nu, w0, len, lane); break;
                default: value_norms_64<VATP_NORM_NONE>(Vu, nu, w0, len, lane); break;
                }
            }
        }

        // stationary operand: 2 column blocks x 8 MFMA steps, 8 bf16 per lane each
        if (qh == 0) {
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
            run.m[0] = run.m[1] = -1e30f;
            run.l[0] = run.l[1] = 0.f;
            run.col[0] = run.col[1] = 0.f;
        }

        // Make the stationary loads complete here, where the compiler can see it: otherwise it
        // waits for them (vmcnt(0)) inside the stage loop, which would also drain the copies in
        // flight that it does not know about.
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int s = 0; s < 8; ++s) asm volatile("" ::"v"(Bf[cb][s]));
        // a neutral pending pair: -inf logits turn into zeros in both epilogues
        Pending<kColsum> pend;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            pend.acc[0][v] = -INFINITY;
            pend.acc[1][v] = -INFINITY;
            if (kColsum) pend.lse[v] = 0.f;
        }
        pend.hist_off[0] = pend.hist_off[1] = 0x80000000u;      // nothing to store for the neutral pair

        // Publish stage t: it is complete once only the copies of younger stages are outstanding.
        // Then the slot freed by stage t-1 (every wavefront is past it now) takes stage t+3.
        auto stage_sync = [&](int t) {
            // (kBand: t is the virtual stage index)
            const int younger = kBand ? min(n_virtual - 1 - t, kAhead - 1) : min(t_end - t, kAhead - 1);
            if (younger == 2) {
                if (extra_copy) wait_copies_then_barrier<10>(); else wait_copies_then_barrier<8>();
            } else if (younger == 1) {
                if (extra_copy) wait_copies_then_barrier<5>(); else wait_copies_then_barrier<4>();
            } else {
                wait_copies_then_barrier<0>();
            }
            if constexpr (kBand) {
                if (issued < n_virtual) issue_copy();
            } else {
                if (t + kAhead <= t_end) copy_stage(t + kAhead, (t + kAhead - t_begin) & (kRing - 1));
            }
        };
        // kBand: this lane's sums over the group's heads of the weights of one stage: [pair][column block][row]
        float group_sum[kBand ? 2 : 1][2][16];
        if constexpr (kBand) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) group_sum[a][cb][v] = 0.f;
        }

        // One stage = two pairs of tiles.  The body is branch-free (the masked variant is a
        // separate instantiation) so that MFMAs and exponentials share one basic block.
        // rowstat: streamed = keys, stationary = queries; a key counts iff key <= query
        // colsum : streamed = queries, stationary = keys
        {
            {
                auto do_stage = [&](int t, auto masked_tag, auto store_tag) __attribute__((always_inline)) {
                    constexpr bool kMasked = decltype(masked_tag)::value;
                    constexpr int kStoreMode = decltype(store_tag)::value;
                    const int slot = kBand ? (cur_v & (kRing - 1)) : ((t - t_begin) & (kRing - 1));
                    const int s0 = t * kSlotRows + kStage * half;   // first streamed row of the sub-stage
                    // the two instantiations must not share a hoisted prefix: the pending pair's
                    // exponentials belong next to this stage's MFMAs (the scale is re-read through
                    // an opaque asm so nothing that uses it can move up)
                    float scale = scale_log2;
                    asm volatile("; stage variant %1" : "+s"(scale) : "n"(kMasked ? 1 : 0));
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        Pending<kColsum> next;
                        const int ar = kStage * half + 32 * kb + n;   // this lane's row of the streamed tile
                        bf16x8 a[8];
#pragma unroll
                        for (int s = 0; s < 8; ++s)
                            a[s] = as_bf16x8(stage[slot][ar * kChunksPerRow + swizzled_chunk(ar, s + 8 * g)]);
                        if (kColsum) {
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) {
                                const float4 x =
                                    *reinterpret_cast<const float4 *>(&lse_stage[slot][kStage * half + 32 * kb + 8 * q4 + 4 * g]);
                                next.lse[4 * q4 + 0] = x.x; next.lse[4 * q4 + 1] = x.y;
                                next.lse[4 * q4 + 2] = x.z; next.lse[4 * q4 + 3] = x.w;
                                if constexpr (kWindow && kGrouped) {      // weights of a group come out divided by its size
#pragma unroll
                                    for (int e = 0; e < 4; ++e) next.lse[4 * q4 + e] += log2_group;
                                }
                            }
                        }
#pragma unroll
                        for (int v = 0; v < 16; ++v) { next.acc[0][v] = 0.f; next.acc[1][v] = 0.f; }
                        if constexpr (kWindow && kColsum) {
                            // byte offset of (first streamed row this lane holds - first window row, its
                            // stationary column); a column past the sequence gets an offset no row can reach
#pragma unroll
                            for (int cb = 0; cb < 2; ++cb) {
                                const int col = w0 + 32 * cb + n;
                                next.hist_off[cb] = col < len ? static_cast<unsigned>(s0 + 32 * kb + 4 * g - q_first) *
                                                                        static_cast<unsigned>(cap * 4) + col * 4
                                                              : 0x80000000u;
                            }
                        }
                        Epilogue<kColsum> epi;
#pragma unroll
                        for (int s = 0; s < 8; ++s) {
                            next.acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], Bf[0][s], next.acc[0], 0, 0, 0);
                            // (the pending pair is the other pair: of the previous virtual stage for kb = 0)
                            epi.template piece<kStoreMode>(2 * s, pend, run, scale, hist_rsrc, cap * 4, group_sum[kBand ? 1 - kb : 0]);
                            next.acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], Bf[1][s], next.acc[1], 0, 0, 0);
                            epi.template piece<kStoreMode>(2 * s + 1, pend, run, scale, hist_rsrc, cap * 4, group_sum[kBand ? 1 - kb : 0]);
                        }
                        epi.finish(pend, run, scale);
                        // keep the pending pair's results inside this block (no sinking past it)
                        if constexpr (kColsum) asm volatile("" : "+v"(run.col[0]), "+v"(run.col[1]));
                        else asm volatile("" : "+v"(run.l[0]), "+v"(run.l[1]), "+v"(run.m[0]), "+v"(run.m[1]));
                        // Issue order asked of the scheduler: a short run of the pending pair's vector
                        // work, then one MFMA per slice of exponentials.  (LDS reads are left to the
                        // scheduler: pinning them makes it drop the whole request.)
                        __builtin_amdgcn_sched_group_barrier(0x002, kLeadValu, 0);
                        sched_two_slots<kSlotValu, kSlotValu>(); sched_two_slots<kSlotValu, kSlotValu>();
                        sched_two_slots<kSlotValu, kSlotValu>(); sched_two_slots<kSlotValu, kSlotValu>();
                        sched_two_slots<kSlotValu, kSlotValu>(); sched_two_slots<kSlotValu, kSlotValu>();
                        sched_two_slots<kSlotValu, kSlotValu>(); sched_two_slots<kSlotValu, kSlotValu>();
                        if constexpr (kMasked) {
                            // -inf above the diagonal of the finished pair and, for streamed
                            // queries, in rows past the end of the sequence
#pragma unroll
                            for (int cb = 0; cb < 2; ++cb) {
                                // lane's stationary index minus the first streamed row it holds
                                const int row0 = s0 + 32 * kb + 4 * g;
                                // (windowed: rows before the window's first query are masked like rows
                                // before the diagonal)
                                const int d0 = kWindow && kColsum ? max((w0 + 32 * cb + n) - row0, q_first - row0)
                                                                  : (w0 + 32 * cb + n) - row0;
                                const int rows_left = len - row0;
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const bool ok = kColsum ? (acc_row(v) >= d0 && acc_row(v) < rows_left)
                                                            : (acc_row(v) <= d0);
                                    next.acc[cb][v] = ok ? next.acc[cb][v] : -INFINITY;
                                }
                            }
                        }
                        pend = next;
                    }
                };
                // Every wavefront walks the same stages (same number of barriers) but spends them
                // differently: full stages, its one diagonal stage, and stages it only waits through.
                // Sub-stage u = t * kHalves + half holds streamed rows 64u .. 64u+63; the one that
                // crosses this wavefront's diagonal is u_diag.  t_first is the first stage whose
                // sub-stage is at or past the diagonal; it is the diagonal itself iff on_diag.
                // (windowed column sums start at the window's first query if that comes later)
                const int u_diag = kWindow && kColsum ? max(w0, q_first) / kStage : w0 / kStage;
                const int du = u_diag - half;
                const int t_first = du < 0 ? 0 : (du + kHalves - 1) / kHalves;
                const bool on_diag = du >= 0 && du % kHalves == 0;
                auto walk = [&](auto store_tag) __attribute__((always_inline)) {
                    int t = t_begin;
                    if (w0 >= len) {
                        for (; t <= t_end; ++t) stage_sync(t);              // no valid stationary row
                    } else if constexpr (!kColsum) {
                        // (a range of keys may end before the diagonal or begin after it)
                        for (; t < t_first && t <= t_end; ++t) { stage_sync(t); do_stage(t, std::false_type{}, store_tag); }
                        if (on_diag && t == t_first && t <= t_end) { stage_sync(t); do_stage(t, std::true_type{}, store_tag); ++t; }
                        for (; t <= t_end; ++t) stage_sync(t);               // keys past the diagonal
                    } else {
                        // last stage whose sub-stage has 64 valid rows: 64u + 63 < len
                        const int t_full_end = (len / kStage - 1 - half + kHalves) / kHalves - 1;
                        for (; t < t_first && t <= t_end; ++t) stage_sync(t);   // queries before the diagonal
                        if (on_diag && t == t_first && t <= t_end) { stage_sync(t); do_stage(t, std::true_type{}, store_tag); ++t; }
                        for (; t <= min(t_full_end, t_end); ++t) { stage_sync(t); do_stage(t, std::false_type{}, store_tag); }
                        for (; t <= t_end; ++t) { stage_sync(t); do_stage(t, std::true_type{}, store_tag); }   // ragged tail
                    }
                    // the last pair still waits for its exponentials
                    Epilogue<kColsum> epi;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        epi.template piece<decltype(store_tag)::value>(i, pend, run, scale_log2, hist_rsrc, cap * 4);
                    epi.finish(pend, run, scale_log2);
                };
                // windowed column sums also leave the attention rows
                if constexpr (kBand) {
                    // every stage of queries once per query head of the group; after the last head the pending
                    // pair is completed (not overlapped with anything: one pair in 2 * group) and the lane's sums
                    // of the stage -- the group means, the weights being divided by the group size -- are stored
                    const int t_full_end = (len / kStage - 1 - half + kHalves) / kHalves - 1;
                    using add_tag = std::integral_constant<int, 2>;
                    for (int t = t_begin; t <= t_end; ++t) {
                        const bool idle = w0 >= len || t < t_first;
                        const bool masked = (on_diag && t == t_first) || t > t_full_end;
                        for (int h = 0; h < group; ++h, ++cur_v) {
                            stage_sync(cur_v);
                            if (idle) continue;
                            if (masked) do_stage(t, std::true_type{}, add_tag{});
                            else do_stage(t, std::false_type{}, add_tag{});
                        }
                        if (idle) continue;
                        Epilogue<kColsum> epi;
#pragma unroll
                        for (int i = 0; i < 16; ++i) epi.template piece<2>(i, pend, run, scale_log2, hist_rsrc, cap * 4, group_sum[1]);
                        epi.finish(pend, run, scale_log2);
#pragma unroll
                        for (int v = 0; v < 16; ++v) { pend.acc[0][v] = -INFINITY; pend.acc[1][v] = -INFINITY; }
#pragma unroll
                        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                            for (int cb = 0; cb < 2; ++cb) {
                                const int col = w0 + 32 * cb + n;
                                const unsigned off = col < len ? static_cast<unsigned>(t * kSlotRows + 32 * kb + 4 * g - q_first) *
                                                                         static_cast<unsigned>(cap * 4) + col * 4
                                                               : 0x80000000u;
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_int(group_sum[kb][cb][v]), hist_rsrc,
                                                                          off + acc_row(v) * (cap * 4), 0, 0);
                                    group_sum[kb][cb][v] = 0.f;
                                }
                            }
                    }
                } else {
                    walk(std::integral_constant<int, (kWindow && kColsum) ? 1 : 0>{});
                }
            }
        }

        if (qh == n_qh - 1) {
        // merge the two lane halves (same stationary column, complementary streamed rows), then,
        // with two sub-stages, the two wavefronts of a column group through LDS
        float fin_m[2], fin_l[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            if (!kColsum) {
                const float m_o = __shfl_xor(run.m[cb], 32), l_o = __shfl_xor(run.l[cb], 32);
                fin_m[cb] = fmaxf(run.m[cb], m_o);
                fin_l[cb] = run.l[cb] * fast_exp2(run.m[cb] - fin_m[cb]) + l_o * fast_exp2(m_o - fin_m[cb]);
            } else {
                fin_m[cb] = 0.f;
                fin_l[cb] = run.col[cb] + __shfl_xor(run.col[cb], 32);
            }
        }
        if constexpr (kHalves == 2) {
            if (half == 1 && g == 0) {
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    merge_buf[0][cw * kWaveCols + 32 * cb + n] = fin_l[cb];
                    if (!kColsum) merge_buf[1][cw * kWaveCols + 32 * cb + n] = fin_m[cb];
                }
            }
            __syncthreads();
            if (half == 0) {
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const float l_o = merge_buf[0][cw * kWaveCols + 32 * cb + n];
                    if (!kColsum) {
                        const float m_o = merge_buf[1][cw * kWaveCols + 32 * cb + n];
                        const float m = fmaxf(fin_m[cb], m_o);
                        fin_l[cb] = fin_l[cb] * fast_exp2(fin_m[cb] - m) + l_o * fast_exp2(m_o - m);
                        fin_m[cb] = m;
                    } else {
                        fin_l[cb] += l_o;
                    }
                }
            }
        }
        if (half == 0 && g == 0) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int idx = w0 + 32 * cb + n;
                if (idx < len) {
                    if constexpr (kSplitKeys)
                        win.lse_part[(static_cast<size_t>(pair % win.n_splits) * n_units + unit) * cap + idx] =
                            fin_m[cb] + __log2f(fin_l[cb]);
                    else if (!kColsum) lse_u[idx] = fin_m[cb] + __log2f(fin_l[cb]);
                    else if (kGrouped && splits > 1)     // partial sum [split, K/V head, cap], mean taken by the merge kernel
                        S[(static_cast<size_t>(split) * (n_units / splits) + unit) * cap + idx] = fin_l[cb];
                    else S[unit * cap + idx] = (kGrouped && !kWindow) ? fin_l[cb] * inv_group : fin_l[cb];   // (windowed groups: weights already divided)
                }
            }
        }
        }
        // every wavefront must be done reading the ring before the next job refills it (all
        // copies have landed by now; the result stores need not have)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
}

}  // namespace

namespace {

constexpr int kSplitStages = 32;       // keys per workgroup of the windowed row statistics: 32 stages of 64

// lse2_j = log2 sum_s 2^(part_s[j]) over the key ranges s that begin at or before row j, for the
// window's queries; the few rows before the window that share its first 64-row stage get 0 (they
// are streamed, masked, by the column-sum pass and must not be NaN).
__global__ __launch_bounds__(256) void merge_split_lse_kernel(const float *__restrict__ lse_part,
                                                              float *__restrict__ lse2, BatchMeta meta,
                                                              int n_heads, int n_units, int cap, int window,
                                                              int n_splits)
{
    const size_t unit = blockIdx.y;
    const int len = meta.len[unit / n_heads];
    const int q_first = max(0, len - 1 - window);
    const int j = q_first / kStage * kStage + blockIdx.x * 256 + threadIdx.x;
    if (j >= len) return;
    float out = 0.f;
    if (j >= q_first) {
        float m = -INFINITY;
        for (int s = 0; s < n_splits && s * kSplitStages * kStage <= j; ++s)
            m = fmaxf(m, lse_part[(static_cast<size_t>(s) * n_units + unit) * cap + j]);
        float l = 0.f;
        for (int s = 0; s < n_splits && s * kSplitStages * kStage <= j; ++s)
            l += exp2f(lse_part[(static_cast<size_t>(s) * n_units + unit) * cap + j] - m);
        out = m + log2f(l);
    }
    lse2[unit * cap + j] = out;
}

}  // namespace

int prefill_window_splits(int cap) { return ((cap + kStage - 1) / kStage + kSplitStages - 1) / kSplitStages; }

bool prefill_mfma_window_fits(int window, int cap, int n_units)
{
    // byte offsets inside one head's [w + 1, cap] matrix of attention rows are 32-bit ...
    if ((static_cast<double>(window) + 1 + kBlockCols) * cap * 4.0 >= 2147483648.0) return false;
    // ... and so is the number of workgroups of the row-statistics launch
    const double n_blocks = (cap + kBlockCols - 1) / kBlockCols;
    const double window_blocks = (window + 1 + kBlockCols - 1) / kBlockCols + 1;
    const double n_qb = window_blocks < n_blocks ? window_blocks : n_blocks;
    return 8.0 * n_qb * prefill_window_splits(cap) * ((n_units + 7) / 8) < 2147483648.0;
}

hipError_t launch_prefill_mfma_window(const void *Q, const void *K, const void *V, float *S, float *nrm, float *lse2,
                                      float *lse_part, int window, float *hist, const BatchMeta &meta,
                                      const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    const int n_blocks = (g.max_len + kBlockCols - 1) / kBlockCols;
    // row statistics per query head, column sums per K/V head (the same units without grouped queries)
    const int kv_units = g.batch * g.n_heads, q_units = kv_units * g.group, q_heads = g.n_heads * g.group;
    const bf16_t *q = static_cast<const bf16_t *>(Q), *k = static_cast<const bf16_t *>(K);
    WindowPass win;
    win.window = window;
    win.hist = hist;
    win.lse_part = lse_part;
    win.split_stages = kSplitStages;
    win.n_splits = ((g.max_len + kStage - 1) / kStage + kSplitStages - 1) / kSplitStages;
    const int window_blocks = (window + 1 + kBlockCols - 1) / kBlockCols + 1;     // blocks a window can straddle
    win.n_qb = window_blocks < n_blocks ? window_blocks : n_blocks;
    hipLaunchKernelGGL((prefill_mfma_kernel<false, 1, true>), dim3(8u * win.n_qb * win.n_splits * ((q_units + 7) / 8)),
                       dim3(256), 0, st, q, k, lse2, S, meta, q_heads, q_units, g.cap, n_blocks, g.scale_log2, win, nullptr,
                       nullptr, 0, g.group, 1);
    const int merge_rows = window + 1 + kStage;
    hipLaunchKernelGGL(merge_split_lse_kernel, dim3((merge_rows + 255) / 256, q_units), dim3(256), 0, st, lse_part, lse2,
                       meta, q_heads, q_units, g.cap, window, win.n_splits);
    const dim3 grid(8u * ((n_blocks + 1) / 2) * ((kv_units + 7) / 8));
    if (g.group > 1)
        hipLaunchKernelGGL((prefill_mfma_kernel<true, 1, true, true>), grid, dim3(256), 0, st, q, k, lse2, S, meta, g.n_heads,
                           kv_units, g.cap, n_blocks, g.scale_log2, win, static_cast<const bf16_t *>(V), nrm, g.norm,
                           g.group, 1);
    else
        hipLaunchKernelGGL((prefill_mfma_kernel<true, 1, true>), grid, dim3(256), 0, st, q, k, lse2, S, meta, g.n_heads,
                           kv_units, g.cap, n_blocks, g.scale_log2, win, static_cast<const bf16_t *>(V), nrm, g.norm, 1, 1);
    return hipGetLastError();
}

namespace {

// S = (1/g) * sum over the splits of the partial column sums a grouped column-sum pass left
__global__ __launch_bounds__(256) void merge_group_partials_kernel(const float *__restrict__ part, float *__restrict__ S,
                                                                   BatchMeta meta, int n_heads, int n_units, int cap,
                                                                   int splits, float inv_group)
{
    const size_t unit = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= meta.len[unit / n_heads]) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += part[(static_cast<size_t>(k) * n_units + unit) * cap + i];
    S[unit * cap + i] = s * inv_group;
}

}  // namespace

hipError_t launch_prefill_mfma(const void *Q, const void *K, const void *V, float *S, float *nrm, float *lse2,
                               float *s_part, bool have_lse, const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    const int n_blocks = (g.max_len + kBlockCols - 1) / kBlockCols;
    const int n_pairs = (n_blocks + 1) / 2;
    const bf16_t *q = static_cast<const bf16_t *>(Q), *k = static_cast<const bf16_t *>(K);
    const bf16_t *v = static_cast<const bf16_t *>(V);
    // One unit per query head in the row-statistics pass, one per K/V head in the column-sum pass (the
    // same count unless query heads share K/V heads).  Two wavefronts per SIMD either way: two
    // 4-wavefront workgroups per compute unit when the grid is large enough to keep pairs of them
    // resident, else 8-wavefront workgroups.
    const int kv_units = g.batch * g.n_heads, q_units = kv_units * g.group;
    const unsigned wg_q = 8u * n_pairs * ((q_units + 7) / 8);
    if (!have_lse) {    // row statistics are computed here unless the caller supplied them
        if (wg_q >= 2u * kComputeUnits)
            hipLaunchKernelGGL((prefill_mfma_kernel<false, 1>), dim3(wg_q), dim3(256), 0, st, q, k, lse2, S, meta,
                               g.n_heads * g.group, q_units, g.cap, n_blocks, g.scale_log2, WindowPass{}, nullptr,
                               nullptr, 0, g.group, 1);
        else
            hipLaunchKernelGGL((prefill_mfma_kernel<false, 2>), dim3(wg_q), dim3(512), 0, st, q, k, lse2, S, meta,
                               g.n_heads * g.group, q_units, g.cap, n_blocks, g.scale_log2, WindowPass{}, nullptr,
                               nullptr, 0, g.group, 1);
    }
    // Grouped column sums: a K/V head's query heads are walked by one workgroup (no partial sums) when that
    // still fills the chip; otherwise they are dealt out to `splits` workgroups -- the smallest divisor of
    // the group size that does -- whose partial sums a small kernel adds.
    int splits = 1;
    if (g.group > 1 && s_part != nullptr)
        for (int s = 1; s <= g.group; ++s)
            if (g.group % s == 0) {
                splits = s;
                if (8u * n_pairs * ((kv_units * s + 7) / 8) >= 2u * kComputeUnits) break;
            }
    const int slots = kv_units * splits;
    const unsigned wg_kv = 8u * n_pairs * ((slots + 7) / 8);
    float *dst = splits > 1 ? s_part : S;
#define VATP_COLSUM(HALVES, GROUPED)                                                                              \
    hipLaunchKernelGGL((prefill_mfma_kernel<true, HALVES, false, GROUPED>), dim3(wg_kv), dim3(256 * HALVES), 0, st, q, k, \
                       lse2, dst, meta, g.n_heads, slots, g.cap, n_blocks, g.scale_log2, WindowPass{}, v, nrm, g.norm,   \
                       g.group, splits)
    if (wg_kv >= 2u * kComputeUnits) {
        if (g.group > 1) VATP_COLSUM(1, true); else VATP_COLSUM(1, false);
    } else {
        if (g.group > 1) VATP_COLSUM(2, true); else VATP_COLSUM(2, false);
    }
#undef VATP_COLSUM
    if (splits > 1)
        hipLaunchKernelGGL(merge_group_partials_kernel, dim3((g.max_len + 255) / 256, kv_units), dim3(256), 0, st, s_part, S,
                           meta, g.n_heads, kv_units, g.cap, splits, 1.f / static_cast<float>(g.group));
    return hipGetLastError();
}

}  // namespace vatp
