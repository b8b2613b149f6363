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


// The same selection with every candidate's key held in registers: one read of S and nrm per row, three
// histogram passes (11, 11 and 10 bits of the key, most significant first) and the ordered emission without
// touching memory again.  A head's rows are dealt to the 16 wavefronts in contiguous ranges of 64 * kPer rows;
// inside a range slot j of lane l is row 64 j + l, so loads are coalesced and a wavefront meets its rows in
// ascending order when it walks its slots.
//   histograms  2048 bins, four copies shared by four wavefronts each (LDS atomics); wide digits, because the
//               first byte of a float's bit pattern (sign and most of the exponent) hardly separates the keys:
//               after the first pass only the keys of one bin -- a few per cent -- take part in the next ones,
//               and a key that does not match the prefix fixed so far costs three instructions
//   emission    every wavefront counts what it keeps, one exclusive scan over the 16 counts gives its first
//               output position and how many rows equal to the threshold it may still admit, and the rows are
//               written in order from ballots -- no workgroup barrier per 1024 rows.
constexpr int kSelBins = 2048, kSelCopies = 4;

// inclusive prefix sum of one value per thread over the 1024 threads of the workgroup (s_tot: 16 words of LDS
// that nothing else touches until the next barrier after the call).  Inside a wavefront the scan runs on DPP
// row shifts (zeros shift in at the row's start) and two broadcasts of a row's last lane to the rows behind it.
__device__ __forceinline__ unsigned block_incl_scan(unsigned v, unsigned *s_tot)
{
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    auto shifted = [](unsigned x, auto ctrl, auto rows) {
        return static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), decltype(ctrl)::value,
                                                                 decltype(rows)::value, 0xf, true));
    };
    using std::integral_constant;
    unsigned x = v;
    x += shifted(x, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{});     // row_shr:1
    x += shifted(x, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{});     // row_shr:2
    x += shifted(x, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{});     // row_shr:4
    x += shifted(x, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{});     // row_shr:8
    x += shifted(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{});     // row_bcast:15 into rows 1 and 3
    x += shifted(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{});     // row_bcast:31 into rows 2 and 3
    if (lane == 63) s_tot[wave] = x;
    __syncthreads();
    unsigned pre = 0;
#pragma unroll
    for (unsigned w = 0; w < kSelThreads / 64; ++w) pre += (w < wave) ? s_tot[w] : 0u;
    return x + pre;
}

template <int kPer>
__global__ __launch_bounds__(kSelThreads) void select_regs_kernel(const float *__restrict__ S,
                                                                  const float *__restrict__ nrm,
                                                                  int32_t *__restrict__ kept_idx, BatchMeta meta,
                                                                  int n_heads, int cap, int cap_out, int n_sink,
                                                                  int recent)
{
    constexpr int kWaves = kSelThreads / 64;
    __shared__ unsigned hist[kSelCopies][kSelBins];
    __shared__ unsigned s_tot[3][kWaves];            // (one set per pass)
    __shared__ unsigned s_keep[kWaves], s_eq[kWaves];
    __shared__ unsigned s_bin, s_k;

    const int b = blockIdx.y, h = blockIdx.x;
    const int n = meta.len[b], B = meta.aux[b];
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const float *Su = S + unit * cap;
    const float *Nu = nrm + unit * cap;
    int32_t *ku = kept_idx + unit * cap_out;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    if (n <= B) {                       // under budget: identity
        for (int r = tid; r < n; r += kSelThreads) ku[r] = r;
        return;
    }
    const int lo = n_sink, hi = n - recent;          // candidates are rows [lo, hi)
    const unsigned k = static_cast<unsigned>(B - n_sink - recent);
    // The protected rows need no decision: the forced prefix goes to the first output positions, the recent
    // window to the last ones.  Only the candidates are dealt to the wavefronts (slot j of this lane is
    // candidate row row0 + 64 j), so every slot of every wavefront but the last one in use holds a candidate.
    for (int i = tid; i < lo; i += kSelThreads) ku[i] = i;
    for (int i = tid; i < recent; i += kSelThreads) ku[B - recent + i] = hi + i;
    const int row0 = lo + wave * 64 * kPer + lane;
    const bool interior = lo + (wave + 1) * 64 * kPer <= hi;      // wavefront-uniform: all of its slots are candidates
    auto is_cand = [&](int j) { return interior || row0 + 64 * j < hi; };

    unsigned key[kPer];
    constexpr int kBatch = kPer < 16 ? kPer : 16;    // loads in flight per thread and array (register budget: 128)
#pragma unroll
    for (int j0 = 0; j0 < kPer; j0 += kBatch) {
        float s_v[kBatch], w_v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {           // all loads of a batch first
            const int r = row0 + 64 * (j0 + u);
            const bool cand = is_cand(j0 + u);
            s_v[u] = cand ? Su[r] : 0.f;
            w_v[u] = cand ? Nu[r] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) key[j0 + u] = __float_as_uint(__fmul_rn(s_v[u], w_v[u]));
    }

    unsigned prefix = 0, mask = 0, kk = k;
    if (k > 0) {
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 21 : pass == 1 ? 10 : 0;
            const unsigned n_bins = pass == 2 ? 1024u : 2048u;
            // (after the first pass only the keys of one bin are left: one copy of the histogram will do)
            const int copies = pass == 0 ? kSelCopies : 1;
            for (int i = tid; i < copies * kSelBins; i += kSelThreads) (&hist[0][0])[i] = 0;
            __syncthreads();
            unsigned *my_hist = hist[pass == 0 ? wave & (kSelCopies - 1) : 0];
            if (interior) {
#pragma unroll
                for (int j = 0; j < kPer; ++j)
                    if ((key[j] & mask) == prefix) atomicAdd(&my_hist[(key[j] >> shift) & (n_bins - 1u)], 1u);
            } else {
#pragma unroll
                for (int j = 0; j < kPer; ++j)
                    if (is_cand(j) && (key[j] & mask) == prefix) atomicAdd(&my_hist[(key[j] >> shift) & (n_bins - 1u)], 1u);
            }
            __syncthreads();
            // thread t owns bins n_bins-1-2t and n_bins-2-2t; find where the count from the top reaches kk
            unsigned c0 = 0, c1 = 0;
            const int top = static_cast<int>(n_bins) - 1 - 2 * tid;
            if (top > 0) {
                for (int c = 0; c < copies; ++c) { c0 += hist[c][top]; c1 += hist[c][top - 1]; }
            }
            const unsigned incl = block_incl_scan(c0 + c1, s_tot[pass]);
            const unsigned excl = incl - (c0 + c1);
            if (excl < kk && kk <= incl) {            // exactly one thread
                if (kk <= excl + c0) { s_bin = static_cast<unsigned>(top); s_k = kk - excl; }
                else { s_bin = static_cast<unsigned>(top - 1); s_k = kk - excl - c0; }
            }
            __syncthreads();
            prefix |= s_bin << shift;
            mask |= (n_bins - 1u) << shift;
            kk = s_k;
            // (s_bin, s_k and the histograms are rewritten only after the next pass's first barrier)
        }
    }
    const unsigned tau = prefix, k_eq = kk;

    // what this wavefront keeps: candidates above the threshold, and its share of those equal to it
    unsigned n_gt = 0, n_eq = 0;
    if (interior) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            n_gt += __popcll(__ballot(k > 0 && key[j] > tau));
            n_eq += __popcll(__ballot(k > 0 && key[j] == tau));
        }
    } else {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const bool cand = is_cand(j);
            n_gt += __popcll(__ballot(cand && k > 0 && key[j] > tau));
            n_eq += __popcll(__ballot(cand && k > 0 && key[j] == tau));
        }
    }
    if (lane == 0) { s_keep[wave] = n_gt; s_eq[wave] = n_eq; }
    __syncthreads();
    unsigned eq_before = 0, out_pos = static_cast<unsigned>(lo);           // (the forced prefix comes first)
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave) {
            const unsigned admit = min(s_eq[w], k_eq - min(k_eq, eq_before));     // equal rows wavefront w may admit
            out_pos += s_keep[w] + admit;
            eq_before += s_eq[w];
        }
    }
    unsigned eq_seen = eq_before;                     // rows equal to the threshold before the current slot
    const unsigned long long below = (1ull << lane) - 1ull;
    if (interior && n_eq == 0) {
        // nothing but candidates, none of them equal to the threshold: a row survives iff its key is larger
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const bool keep = k > 0 && key[j] > tau;
            const unsigned long long keep_mask = __ballot(keep);
            if (keep) ku[out_pos + __popcll(keep_mask & below)] = row0 + 64 * j;
            out_pos += __popcll(keep_mask);
        }
    } else {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const bool cand = is_cand(j);
            const bool iseq = cand && k > 0 && key[j] == tau;
            const unsigned long long eq_mask = __ballot(iseq);
            const bool keep = cand && k > 0 && (key[j] > tau || (iseq && eq_seen + __popcll(eq_mask & below) < k_eq));
            const unsigned long long keep_mask = __ballot(keep);
            if (keep) ku[out_pos + __popcll(keep_mask & below)] = row0 + 64 * j;
            out_pos += __popcll(keep_mask);
            eq_seen += __popcll(eq_mask);
        }
    }
}

}  // namespace

hipError_t launch_select(const float *S, const float *nrm, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    dim3 grid(g.n_heads, g.batch), block(kSelThreads);
    // rows of the longest sequence before the prune (meta.len), per thread of the 1024: keys stay in registers
    // up to 64 per thread; longer heads take the kernel that re-reads S and nrm in every pass
    int longest = 0;
    for (int b = 0; b < g.batch; ++b) longest = meta.len[b] > longest ? meta.len[b] : longest;
#define VATP_SEL(PER)                                                                                          \
    hipLaunchKernelGGL(select_regs_kernel<PER>, grid, block, 0, st, S, nrm, kept_idx, meta, g.n_heads, g.cap, \
                       g.cap_out, g.n_sink, g.recent)
    if (longest <= 4 * kSelThreads) VATP_SEL(4);
    else if (longest <= 16 * kSelThreads) VATP_SEL(16);
    else if (longest <= 32 * kSelThreads) VATP_SEL(32);
    else if (longest <= 64 * kSelThreads) VATP_SEL(64);
    else
        hipLaunchKernelGGL(select_kernel, grid, block, 0, st, S, nrm, kept_idx, meta, g.n_heads, g.cap, g.cap_out,
                           g.n_sink, g.recent);
#undef VATP_SEL
    return hipGetLastError();
}

}  // namespace vatp
