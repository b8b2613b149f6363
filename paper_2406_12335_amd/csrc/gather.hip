// Compaction of the surviving rows (paper Fig. 2: the least important token's K/V row is
// removed; Implementation Details appendix: a fixed budget of rows per head remains).
//
// HBM-bound row gather, out of place, order preserving: output row o of a unit receives
// source row kept[o]; a row of head_dim elements moves as 16 bytes per lane, a group of
// lanes per row, so consecutive surviving rows make one contiguous span on both sides.
//
// Two ways to learn kept[]:
//   kFromIndex  the selection kernel has already written kept_idx;
//   kEvictOne   exactly one row leaves (a decode step at steady state, n = B + 1): every
//               workgroup finds the evicted row itself -- the candidate with the smallest
//               importance S*nrm, the highest index among equals, which is the complement
//               of "largest first, lower index wins" -- and writes its share of kept_idx.
#include "vatp_device.h"

namespace vatp {

namespace {

constexpr int kGatherRows = 64;    // output rows per workgroup

template <typename T, int D, bool kEvictOne, bool kStream>
__global__ __launch_bounds__(256) void gather_kernel(
    const T *__restrict__ K, const T *__restrict__ V, const float *__restrict__ S,
    const float *__restrict__ nrm, const int32_t *__restrict__ pos, T *__restrict__ K_out,
    T *__restrict__ V_out, float *__restrict__ S_out, float *__restrict__ nrm_out,
    int32_t *__restrict__ pos_out, int32_t *kept_idx, BatchMeta meta, int n_heads, int cap,
    int cap_out, int n_sink, int recent)
{
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = 256 / kLanesPerRow;

    __shared__ unsigned long long s_min[4];
    __shared__ int s_src[kGatherRows];

    const int b = blockIdx.z, h = blockIdx.y;
    const int n = meta.len[b], B = meta.aux[b];
    const int n_keep = n < B ? n : B;
    const int o0 = blockIdx.x * kGatherRows;
    if (o0 >= n_keep) return;
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const float *Su = S + unit * cap;
    const float *Nu = nrm + unit * cap;
    int32_t *ku = kept_idx + unit * cap_out;
    const int tid = threadIdx.x;

    if constexpr (kEvictOne) {
        int evicted = n;                                   // n <= B: nothing leaves
        if (n > B) {
            const int lo = n_sink, hi = n - recent;
            // minimise (importance bits, ~row): smallest importance, highest row among equals
            unsigned long long best = ~0ull;
            for (int r = lo + tid; r < hi; r += 256) {
                const unsigned key = __float_as_uint(__fmul_rn(Su[r], Nu[r]));
                const unsigned long long c = (static_cast<unsigned long long>(key) << 32) |
                                             static_cast<unsigned>(~static_cast<unsigned>(r));
                best = c < best ? c : best;
            }
            best = wave_min_u64(best);
            if ((tid & 63) == 0) s_min[tid >> 6] = best;
            __syncthreads();
            best = s_min[0];
#pragma unroll
            for (int w = 1; w < 4; ++w) best = s_min[w] < best ? s_min[w] : best;
            evicted = static_cast<int>(~static_cast<unsigned>(best & 0xffffffffull));
        }
        if (tid < kGatherRows) {
            const int o = o0 + tid;
            const int src = o + (o >= evicted ? 1 : 0);
            s_src[tid] = src;
            if (o < n_keep) ku[o] = src;
        }
    } else {
        if (tid < kGatherRows) {
            const int o = o0 + tid;
            s_src[tid] = (o < n_keep) ? ku[o] : 0;
        }
    }
    __syncthreads();

    if (tid < kGatherRows) {
        const int o = o0 + tid;
        if (o < n_keep) {
            const int src = s_src[tid];
            S_out[unit * cap_out + o] = Su[src];
            nrm_out[unit * cap_out + o] = Nu[src];
            if (pos_out) pos_out[unit * cap_out + o] = pos[unit * cap + src];
        }
    }

    const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
    const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * D);
    uint4 *Ko = reinterpret_cast<uint4 *>(K_out + unit * cap_out * D);
    uint4 *Vo = reinterpret_cast<uint4 *>(V_out + unit * cap_out * D);
    const int sub = tid % kLanesPerRow;
    const int rloc = tid / kLanesPerRow;
#pragma unroll
    for (int pass = 0; pass < kGatherRows / kRowsPerPass; ++pass) {
        const int ol = pass * kRowsPerPass + rloc;
        const int o = o0 + ol;
        if (o < n_keep) {
            const size_t src = static_cast<size_t>(s_src[ol]) * kLanesPerRow + sub;
            const size_t dst = static_cast<size_t>(o) * kLanesPerRow + sub;
            const uint4 kr = load_rows<kStream>(Ku + src);
            const uint4 vr = load_rows<kStream>(Vu + src);
            store_rows<kStream>(Ko + dst, kr);
            store_rows<kStream>(Vo + dst, vr);
        }
    }
}

// History-window scores (Eq. 3): after the prompt has been pruned, the window's attention rows
// follow the surviving tokens.  hist_in holds a_i^j at [j - j_first][i] for the prompt's last
// rows-1 queries j >= j_first and keys i <= j (what the prompt pass stored; everything else is
// undefined and reads as 0 here); hist_out, a ring of `rows` rows in which query j sits in row
// j mod rows, receives column kept[o] as column o, and surviving row o is given history column o.
constexpr int kHistRowsPerBlock = 8;     // ring rows per workgroup of the history gather

__global__ __launch_bounds__(256) void hist_gather_kernel(const float *__restrict__ hist_in,
                                                          const int32_t *__restrict__ kept_idx,
                                                          float *__restrict__ hist_out, int32_t *__restrict__ hid_out,
                                                          int32_t *__restrict__ free_out, BatchMeta meta, int n_heads,
                                                          int cap, int cap_out, int cap_hist, int rows)
{
    const size_t unit = blockIdx.y;
    const int b = static_cast<int>(unit / n_heads);
    const int n = meta.len[b], B = meta.aux[b];
    const int n_keep = n < B ? n : B;
    const int o = blockIdx.x * 256 + threadIdx.x;
    const int s0 = blockIdx.z * kHistRowsPerBlock;
    if (blockIdx.x == 0 && blockIdx.z == 0 && threadIdx.x == 0) free_out[unit] = n_keep;
    if (o >= n_keep) return;
    const int src = kept_idx[unit * cap_out + o];
    if (blockIdx.z == 0) hid_out[unit * cap_out + o] = o;
    const int q_first = max(0, n - (rows - 1));            // first query of the window (w + 1 = rows - 1 of them)
    float val[kHistRowsPerBlock];
#pragma unroll
    for (int u = 0; u < kHistRowsPerBlock; ++u) {          // all loads first, then the stores
        const int s = s0 + u;
        const int j = q_first + (s - q_first % rows + rows) % rows;     // the window's query kept in ring row s
        const bool defined = s < rows && j < n && src <= j;
        val[u] = defined ? hist_in[(unit * (rows - 1) + (j - q_first)) * static_cast<size_t>(cap) + src] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kHistRowsPerBlock; ++u)
        if (s0 + u < rows) hist_out[(unit * rows + s0 + u) * static_cast<size_t>(cap_hist) + o] = val[u];
}

// Low-order parts of the survivors' windowed scores after the prompt prune: the survivor's column of the ring is
// summed in two floats (ring rows in order) and s_lo_out receives that sum minus the score the selection copied,
// so that S_out + s_lo_out carries the window's weights exactly (to two floats) into the decode steps.
__global__ __launch_bounds__(256) void window_low_part_kernel(const float *__restrict__ hist_out,
                                                              const float *__restrict__ S_out, float *__restrict__ s_lo_out,
                                                              BatchMeta meta, int n_heads, int cap_out, int cap_hist, int rows)
{
    const size_t unit = blockIdx.y;
    const int b = static_cast<int>(unit / n_heads);
    const int n = meta.len[b], B = meta.aux[b];
    const int n_keep = n < B ? n : B;
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= n_keep) return;
    float hi = 0.f, lo = 0.f;
    for (int s0 = 0; s0 < rows; s0 += 8) {
        float val[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            val[u] = s0 + u < rows ? hist_out[(unit * rows + s0 + u) * static_cast<size_t>(cap_hist) + o] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) two_float_add(hi, lo, val[u]);
    }
    s_lo_out[unit * cap_out + o] = __fadd_rn(__fsub_rn(hi, S_out[unit * cap_out + o]), lo);
}

}  // namespace

hipError_t launch_gather(int dtype, int head_dim, bool evict_one,
                         const void *K, const void *V, const float *S, const float *nrm,
                         const int32_t *pos, void *K_out, void *V_out, float *S_out,
                         float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;       // max_len: largest surviving row count
    dim3 grid((g.max_len + kGatherRows - 1) / kGatherRows, g.n_heads, g.batch), block(256);
#define VATP_GA(T, D, E)                                                                         \
    do {                                                                                         \
        if (g.stream) VATP_GA_S(T, D, E, true);                                                  \
        else VATP_GA_S(T, D, E, false);                                                          \
    } while (0)
#define VATP_GA_S(T, D, E, STREAM)                                                                    \
    hipLaunchKernelGGL((gather_kernel<T, D, E, STREAM>), grid, block, 0, st, static_cast<const T *>(K), \
                       static_cast<const T *>(V), S, nrm, pos, static_cast<T *>(K_out),          \
                       static_cast<T *>(V_out), S_out, nrm_out, pos_out, kept_idx, meta,         \
                       g.n_heads, g.cap, g.cap_out, g.n_sink, g.recent)
#define VATP_GA2(T, D) do { if (evict_one) VATP_GA(T, D, true); else VATP_GA(T, D, false); } while (0)
    if (dtype == VATP_F32 && head_dim == 64) VATP_GA2(float, 64);
    else if (dtype == VATP_F32) VATP_GA2(float, 128);
    else if (head_dim == 64) VATP_GA2(bf16_t, 64);
    else VATP_GA2(bf16_t, 128);
#undef VATP_GA2
#undef VATP_GA
#undef VATP_GA_S
    return hipGetLastError();
}

}  // namespace vatp

namespace vatp {

hipError_t launch_hist_gather(const float *hist_in, const int32_t *kept_idx, float *hist_out, int32_t *hid_out,
                              int32_t *free_out, const float *S_out, float *s_lo_out, int rows, int cap_hist,
                              const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    const unsigned units = static_cast<unsigned>(g.batch) * g.n_heads;
    const int max_keep = g.max_len > 0 ? g.max_len : 1;       // max_len: largest surviving row count
    hipLaunchKernelGGL(hist_gather_kernel,
                       dim3((max_keep + 255) / 256, units, (rows + kHistRowsPerBlock - 1) / kHistRowsPerBlock), dim3(256), 0,
                       st, hist_in, kept_idx,
                       hist_out, hid_out, free_out, meta, g.n_heads, g.cap, g.cap_out, cap_hist, rows);
    hipLaunchKernelGGL(window_low_part_kernel, dim3((max_keep + 255) / 256, units), dim3(256), 0, st, hist_out, S_out,
                       s_lo_out, meta, g.n_heads, g.cap_out, cap_hist, rows);
    return hipGetLastError();
}

}  // namespace vatp
