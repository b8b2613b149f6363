// Budgeted per-head selection (paper: Eq. 4 importance; forced prefix of the Attention
// Sink Tokens paragraph; budget and local window of the Implementation Details appendix).
//
// One workgroup per (batch, head) unit.  Importance I = S * nrm is a non-negative float32,
// so its bit pattern orders like an unsigned integer.  The B-F-R largest candidates are
// found by a most-significant-byte-first radix select: four passes, each a 256-bin
// histogram in LDS (LDS atomics only) over the candidates that match the prefix fixed so
// far.  The result is the threshold pattern tau and the number k_eq of candidates equal
// to tau that still fit; an ordered sweep then emits the surviving rows in ascending
// order, admitting the first k_eq rows equal to tau (lower index wins a tie).
#include "vatp_device.h"

namespace vatp {

namespace {

constexpr int kSelThreads = 1024;

__device__ __forceinline__ unsigned block_excl_scan_flag(bool f, unsigned *s_tot, unsigned &total)
{
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long bal = __ballot(f);
    const unsigned within = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_tot[wave] = __popcll(bal);
    __syncthreads();
    unsigned pre = 0, tot = 0;
#pragma unroll
    for (unsigned w = 0; w < kSelThreads / 64; ++w) {
        const unsigned v = s_tot[w];
        pre += (w < wave) ? v : 0u;
        tot += v;
    }
    __syncthreads();
    total = tot;
    return pre + within;
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float *__restrict__ S,
                                                             const float *__restrict__ nrm,
                                                             int32_t *__restrict__ kept_idx,
                                                             BatchMeta meta, int n_heads, int cap,
                                                             int cap_out, int n_sink, int recent)
{
    __shared__ unsigned hist[256];
    __shared__ unsigned s_tot[kSelThreads / 64];
    __shared__ unsigned s_bin, s_k;

    const int b = blockIdx.y, h = blockIdx.x;
    const int n = meta.len[b], B = meta.aux[b];
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const float *Su = S + unit * cap;
    const float *Nu = nrm + unit * cap;
    int32_t *ku = kept_idx + unit * cap_out;
    const int tid = threadIdx.x;

    if (n <= B) {                       // under budget: identity
        for (int r = tid; r < n; r += kSelThreads) ku[r] = r;
        return;
    }
    const int lo = n_sink, hi = n - recent;          // candidates are rows [lo, hi)
    const unsigned k = static_cast<unsigned>(B - n_sink - recent);

    unsigned prefix = 0, mask = 0, kk = k;
    if (k > 0) {
        for (int pass = 3; pass >= 0; --pass) {
            const int shift = pass * 8;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int r = lo + tid; r < hi; r += kSelThreads) {
                const unsigned key = __float_as_uint(__fmul_rn(Su[r], Nu[r]));
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid < 64) {
                // lane L owns bins 255-4L .. 252-4L; find where the count from the top reaches kk
                unsigned c[4], tot = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) { c[i] = hist[255 - (4 * tid + i)]; tot += c[i]; }
                unsigned incl = tot;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const unsigned v = __shfl_up(incl, off);
                    if (tid >= off) incl += v;
                }
                unsigned cum = incl - tot;
                if (cum < kk && kk <= incl) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (cum < kk && kk <= cum + c[i]) { s_bin = 255 - (4 * tid + i); s_k = kk - cum; }
                        cum += c[i];
                    }
                }
            }
            __syncthreads();
            prefix |= s_bin << shift;
            mask |= 255u << shift;
            kk = s_k;
            __syncthreads();
        }
    }
    const unsigned tau = prefix, k_eq = kk;

    unsigned run_out = 0, run_eq = 0;
    for (int base = 0; base < n; base += kSelThreads) {
        const int r = base + tid;
        const bool valid = r < n;
        const bool cand = valid && r >= lo && r < hi;
        const unsigned key = cand ? __float_as_uint(__fmul_rn(Su[r], Nu[r])) : 0u;
        const bool iseq = cand && k > 0 && key == tau;
        unsigned eq_total;
        const unsigned eq_excl = block_excl_scan_flag(iseq, s_tot, eq_total);
        const bool keep = valid && (!cand || (k > 0 && (key > tau || (iseq && run_eq + eq_excl < k_eq))));
        unsigned keep_total;
        const unsigned out_excl = block_excl_scan_flag(keep, s_tot, keep_total);
        if (keep) ku[run_out + out_excl] = r;
        run_out += keep_total;
        run_eq += eq_total;
    }
}

}  // namespace

hipError_t launch_select(const float *S, const float *nrm, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    dim3 grid(g.n_heads, g.batch), block(kSelThreads);
    hipLaunchKernelGGL(select_kernel, grid, block, 0, st, S, nrm, kept_idx, meta, g.n_heads,
                       g.cap, g.cap_out, g.n_sink, g.recent);
    return hipGetLastError();
}

}  // namespace vatp
