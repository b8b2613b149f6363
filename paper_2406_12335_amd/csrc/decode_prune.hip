// Second launch of the fused decode-and-evict step: finishes the softmax of the new query,
// adds the attention weights to the running scores (paper Eq. 2, incrementally), finds the one
// row per head that has to leave (smallest S * nrm among the rows that are neither sink nor
// recent, Eq. 4; the highest index among equals) and brings the other cache set up to date.
//
// The two cache sets alternate as input and output.  After a step that removed input row e,
// the old input set still agrees with the new state in its rows 0 .. e-1, so the next step
// (which writes into it) only has to rewrite rows from min(synced, e') on, where e' is its own
// evicted row.  The per-head count `synced` travels in a small device array.  Rows that have
// just left the recent window carry the smallest accumulated scores, so in practice only about
// `recent` rows move per step instead of the whole cache; the scores themselves change in
// every row and are rewritten in full.
//
// Grid: (units, G).  Each of a head's G workgroups repeats the cheap part (12 bytes per row
// from L2: logit, S, nrm) to learn the evicted row by itself, then takes a 1/G share of the
// stores, so the launch needs no exchange between workgroups and no second pass.
//
// Arithmetic is the same, operation for operation, as decode_finish_kernel followed by the
// evict-one gather, so both routes give identical bits.
#include "vatp_device.h"

namespace vatp {

namespace {

constexpr int kThreads = 512;

template <typename T, int D, int kMaxG>
__global__ __launch_bounds__(kThreads) void decode_prune_kernel(
    const T *__restrict__ K, const T *__restrict__ V, const float *__restrict__ S,
    const float *__restrict__ nrm, const int32_t *__restrict__ pos, T *__restrict__ K_out,
    T *__restrict__ V_out, float *__restrict__ S_out, float *__restrict__ nrm_out,
    int32_t *__restrict__ pos_out, int32_t *__restrict__ kept_idx, const int32_t *__restrict__ synced_in,
    int32_t *__restrict__ synced_out, const float *__restrict__ ws_logit, const float2 *__restrict__ ws_part,
    const float *__restrict__ ws_out, float *__restrict__ out, WindowArgs win, BatchMeta meta, int n_heads,
    int cap, int cap_out, int chunks_alloc, int n_sink, int recent, int group, int stream)
{
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = kThreads / kLanesPerRow;

    __shared__ unsigned long long s_min[kThreads / 64];

    // workgroups go to the 8 XCDs round-robin by linear id = unit + units * g: with the unit in the fast
    // dimension a head's G workgroups meet in one XCD's L2 (unit count a multiple of 8), where the rows
    // they all scan are fetched once
    const size_t unit = blockIdx.x;
    const int g = blockIdx.y, G = gridDim.y;
    const int b = static_cast<int>(unit / n_heads);
    const int n0 = meta.len[b], n = n0 + 1, B = meta.aux[b];
    const int n_keep = n < B ? n : B;
    const int tid = threadIdx.x;
    const float *Su = S + unit * cap;
    const float *Nu = nrm + unit * cap;
    const float *Lu = ws_logit + unit * group * cap;       // the group's logits: query head i at Lu + i * cap

    const int synced = synced_in[unit];
    const int lo = n_sink, hi = n - recent;                // rows [lo, hi) may leave

    // history window (Eq. 3): the ring row this step writes, the one that leaves the window, and
    // the column of every row (the appended row takes the free column and has no past)
    const bool windowed = win.hist != nullptr;
    const int step = windowed ? win.step[b] : 0;
    float *h_write = windowed ? win.hist + (unit * win.rows + step % win.rows) * static_cast<size_t>(win.cap_hist) : nullptr;
    const float *h_leave =
        windowed ? win.hist + (unit * win.rows + (step + 1) % win.rows) * static_cast<size_t>(win.cap_hist) : nullptr;
    const int new_col = windowed ? win.free_in[unit] : 0;
    auto column = [&](int r) { return r == n0 ? new_col : win.hid[unit * cap + r]; };
    auto leaving = [&](int r) { return windowed && r != n0 ? h_leave[column(r)] : 0.f; };
    auto low_part = [&](int r) { return windowed && r != n0 ? win.s_lo[unit * cap + r] : 0.f; };

    // the unprotected rows this thread looks at (logit, old score, norm), requested before the
    // denominator is known so that both round trips to memory overlap
    constexpr int kScan = kMaxG > 8 ? 1 : 4;                 // rows per thread and round trip (each brings kMaxG logits)
    float t_r[kScan][kMaxG], s_r[kScan], w_r[kScan], x_r[kScan], l_r[kScan];
#pragma unroll
    for (int u = 0; u < kScan; ++u) {
        const int r = lo + tid + u * kThreads;
        const bool ok = n > B && r < hi;
        load_group_logits<kMaxG>(t_r[u], Lu, cap, group, r, ok);
        s_r[u] = ok && r != n0 ? Su[r] : 0.f;
        w_r[u] = ok ? Nu[r] : 0.f;
        x_r[u] = ok ? leaving(r) : 0.f;
        l_r[u] = ok ? low_part(r) : 0.f;
    }

    // log2 of the softmax denominator of every query head of the group from the chunk statistics
    const int n_chunks = (n + kDecodeChunk - 1) / kDecodeChunk;
    const float2 *part = ws_part + unit * group * chunks_alloc;
    float lse2[kMaxG];
    merge_group_stats<kMaxG>(part, chunks_alloc, group, n_chunks, lse2);

    // new score from the old one, this step's attention weight and (windowed) the weight that leaves the
    // window: accumulated scores are one fp32 addition; windowed scores are carried in two floats (window_update),
    // so that adding a weight and subtracting the same float w+1 steps later leaves no residue behind
    auto combine = [&](float s_old, float lo_old, float p, float gone, float &lo_new) {
        if (!windowed) { lo_new = 0.f; return s_old + p; }
        float hi = s_old, lo = lo_old;
        window_update(hi, lo, gone, p);
        lo_new = lo;
        return hi;
    };
    float unused_lo;

    // the row that leaves: minimise (importance bits, ~row) over the unprotected rows
    int evicted = n;                                       // n <= B: nothing leaves
    if (n > B) {
        unsigned long long best = ~0ull;
        auto consider = [&](int r, float score, float w) {
            const unsigned key = __float_as_uint(__fmul_rn(score, w));
            const unsigned long long c =
                (static_cast<unsigned long long>(key) << 32) | static_cast<unsigned>(~static_cast<unsigned>(r));
            best = c < best ? c : best;
        };
#pragma unroll
        for (int u = 0; u < kScan; ++u) {
            const int r = lo + tid + u * kThreads;
            if (r < hi) consider(r, combine(s_r[u], l_r[u], group_weight<kMaxG>(t_r[u], lse2, group), x_r[u], unused_lo), w_r[u]);
        }
        // further rows, four per thread at a time: loads first, then the arithmetic
        for (int r0 = lo + tid + kScan * kThreads; r0 < hi; r0 += kScan * kThreads) {
            float t4[kScan][kMaxG], s4[kScan], w4[kScan], x4[kScan], l4[kScan];
#pragma unroll
            for (int u = 0; u < kScan; ++u) {
                const int r = r0 + u * kThreads;
                const bool ok = r < hi;
                load_group_logits<kMaxG>(t4[u], Lu, cap, group, r, ok);
                s4[u] = ok && r != n0 ? Su[r] : 0.f;
                w4[u] = ok ? Nu[r] : 0.f;
                x4[u] = ok ? leaving(r) : 0.f;
                l4[u] = ok ? low_part(r) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kScan; ++u) {
                const int r = r0 + u * kThreads;
                if (r < hi) consider(r, combine(s4[u], l4[u], group_weight<kMaxG>(t4[u], lse2, group), x4[u], unused_lo), w4[u]);
            }
        }
        best = wave_min_u64(best);
        if ((tid & 63) == 0) s_min[tid >> 6] = best;
        __syncthreads();
        best = s_min[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) best = s_min[w] < best ? s_min[w] : best;
        evicted = static_cast<int>(~static_cast<unsigned>(best & 0xffffffffull));
    }

    // scores and source indices of this workgroup's share of the surviving rows
    {
        const int share = (n_keep + G - 1) / G;
        const int o_end = min(n_keep, (g + 1) * share);
        for (int o0 = g * share + tid; o0 < o_end; o0 += kScan * kThreads) {
            float t4[kScan][kMaxG], s4[kScan], x4[kScan], l4[kScan];
            int c4[kScan];
#pragma unroll
            for (int u = 0; u < kScan; ++u) {           // loads first, then the arithmetic and the stores
                const int o = o0 + u * kThreads;
                const int src = o + (o >= evicted ? 1 : 0);
                const bool ok = o < o_end;
                load_group_logits<kMaxG>(t4[u], Lu, cap, group, src, ok);
                s4[u] = ok && src != n0 ? Su[src] : 0.f;
                x4[u] = ok ? leaving(src) : 0.f;
                l4[u] = ok ? low_part(src) : 0.f;
                c4[u] = ok && windowed ? column(src) : 0;
            }
#pragma unroll
            for (int u = 0; u < kScan; ++u) {
                const int o = o0 + u * kThreads;
                if (o >= o_end) continue;
                const float p = group_weight<kMaxG>(t4[u], lse2, group);
                float lo_new;
                S_out[unit * cap_out + o] = combine(s4[u], l4[u], p, x4[u], lo_new);
                if (windowed) win.s_lo_out[unit * cap_out + o] = lo_new;
                if (kept_idx) kept_idx[unit * cap_out + o] = o + (o >= evicted ? 1 : 0);
                if (windowed) h_write[c4[u]] = p;
            }
        }
    }
    if (windowed && g == 0) {
        // the appended row has received nothing in the steps before this one: clear its column in every
        // ring row but the one written above and the one that leaves (rewritten in full by the next step)
        for (int s = tid; s < win.rows; s += kThreads)
            if (s != step % win.rows && s != (step + 1) % win.rows)
                win.hist[(unit * win.rows + s) * static_cast<size_t>(win.cap_hist) + new_col] = 0.f;
        if (tid == 0) {
            win.hid[unit * cap + n0] = new_col;
            win.free_out[unit] = evicted < n ? column(evicted) : n;     // a fresh column while the cache grows
        }
    }

    // rows of the other set that are out of date: from the first row in which it differs from
    // the input set, or from the evicted row if that comes earlier
    const int first = min(synced, evicted);
    if (g == 0 && tid == 0) synced_out[unit] = evicted;
    {
        const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
        const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * D);
        uint4 *Ko = reinterpret_cast<uint4 *>(K_out + unit * cap_out * D);
        uint4 *Vo = reinterpret_cast<uint4 *>(V_out + unit * cap_out * D);
        const int sub = tid % kLanesPerRow;
        const int rloc = tid / kLanesPerRow;
        for (int o = first + g * kRowsPerPass + rloc; o < n_keep; o += G * kRowsPerPass) {
            const int src = o + (o >= evicted ? 1 : 0);
            uint4 kr, vr;
            if (stream) {       // (uniform: the whole call either streams or does not)
                kr = load_stream(Ku + static_cast<size_t>(src) * kLanesPerRow + sub);
                vr = load_stream(Vu + static_cast<size_t>(src) * kLanesPerRow + sub);
                store_stream(Ko + static_cast<size_t>(o) * kLanesPerRow + sub, kr);
                store_stream(Vo + static_cast<size_t>(o) * kLanesPerRow + sub, vr);
            } else {
                kr = Ku[static_cast<size_t>(src) * kLanesPerRow + sub];
                vr = Vu[static_cast<size_t>(src) * kLanesPerRow + sub];
                Ko[static_cast<size_t>(o) * kLanesPerRow + sub] = kr;
                Vo[static_cast<size_t>(o) * kLanesPerRow + sub] = vr;
            }
            if (sub == 0) {
                nrm_out[unit * cap_out + o] = Nu[src];
                if (pos_out) pos_out[unit * cap_out + o] = pos[unit * cap + src];
                if (windowed) win.hid_out[unit * cap_out + o] = column(src);
            }
        }
    }

    // attention output of the new token (optional), per query head: the chunks' partial sums on a common maximum
    if (out && g == 0)
        merge_group_outputs(out + unit * group * D, ws_out + unit * group * chunks_alloc * D, part, chunks_alloc, n_chunks,
                            group, D, kThreads);
}

// The whole step in one launch, one workgroup of 16 wavefronts per head: logits of the new query
// over the head's rows (they stay in LDS), softmax statistics, new scores, the evicted row, and
// the rows of the other cache set that are out of date.  Used when every head's rows fit the LDS
// buffer; no workspace traffic and no second launch.  Logits and per-chunk statistics are formed by
// the same functions as in decode_logits_kernel (dot_16_bytes, group_all_reduce, chunk_stats_64x2 on
// 128-row chunks), so the result has the same bits as the two-launch route.
//
// Rows are dealt to threads from the END of the cache: load slot u of thread (rloc, sub) is row
// n-1 - (u * rows_per_pass + rloc).  The row that leaves is almost always the one at the edge of the recent
// window, e* = n - recent - 1 (it has just lost the window's protection and has collected the least
// attention), and then exactly the rows behind it move one position down in the other set.  Those rows are
// the first slots of every thread: their V rows, norms and positions are the first loads of the kernel,
// their K rows the first of the stream, and they are stored -- to the positions the guess e* implies -- as
// soon as they have arrived, while the rest of the head is still streaming in, instead of in a burst at the
// end.  When the real evicted row e turns out to lie before e*, what was stored is still right (rows behind
// e* move down by one either way); row e* itself, which the guess skipped, is then stored to e* - 1 from the
// registers that still hold it, and the rows between e and e* are copied the ordinary way.
constexpr int kOneThreads = 1024;
constexpr int kOneMaxRows = 2048;                          // logits, old scores and norms kept in LDS (24 KiB)

template <typename T, int D, bool kStream>
__global__ __launch_bounds__(kOneThreads) void decode_prune_one_kernel(
    const T *__restrict__ q, const T *__restrict__ k_new, const T *__restrict__ v_new, T *__restrict__ K,
    T *__restrict__ V, const float *__restrict__ S, float *__restrict__ nrm, int32_t *__restrict__ pos,
    T *__restrict__ K_out, T *__restrict__ V_out, float *__restrict__ S_out, float *__restrict__ nrm_out,
    int32_t *__restrict__ pos_out, int32_t *__restrict__ kept_idx, const int32_t *__restrict__ synced_in,
    int32_t *__restrict__ synced_out, BatchMeta len_pos, BudgetList budget, int n_heads, int cap, int cap_out,
    int n_sink, int recent, float scale_log2, int norm)
{
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = kOneThreads / kLanesPerRow;
    constexpr int kGroup = 16;                             // row loads in flight per thread: 1024 rows per round trip
    constexpr int kWaves = kOneThreads / 64;
    constexpr int kPre = kOneMaxRows / kOneThreads;        // rows of S and nrm a thread brings in
    // rows requested ahead of the eviction: the last kSpecRows of the cache (>= 128), kSpecSlots per thread
    constexpr int kSpecSlots = kRowsPerPass >= 64 ? 2 : 128 / kRowsPerPass, kSpecRows = kSpecSlots * kRowsPerPass;
    static_assert(kSpecSlots <= kGroup, "the speculative rows are slots of the first round trip");

    __shared__ float s_logit[kOneMaxRows];
    __shared__ float s_score[kOneMaxRows];                 // old scores (0 for the appended row)
    __shared__ float s_norm[kOneMaxRows];
    __shared__ float2 s_part[kOneMaxRows / kDecodeChunk];
    __shared__ float s_new_norm;
    __shared__ unsigned long long s_min[kWaves];

    const size_t unit = blockIdx.x;
    const int b = static_cast<int>(unit / n_heads);
    const int n0 = len_pos.len[b], n = n0 + 1, B = budget.v[b];
    const int n_keep = n < B ? n : B;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = tid % kLanesPerRow, rloc = tid / kLanesPerRow;
    const float *Su = S + unit * cap;
    float *Nu = nrm + unit * cap;
    const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
    const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * D);
    const uint4 *knew = reinterpret_cast<const uint4 *>(k_new + unit * D);
    const uint4 *vnew = reinterpret_cast<const uint4 *>(v_new + unit * D);

    // the row expected to leave (n > B: there are candidates, so n - recent - 1 >= n_sink), and the first of
    // the rows that are stored ahead of the decision
    const int e_star = n > B ? n - recent - 1 : n;
    const int spec_lo = max(max(n - recent - 1, n - kSpecRows), 0);
    uint4 *Ko = reinterpret_cast<uint4 *>(K_out + unit * cap_out * D);
    uint4 *Vo = reinterpret_cast<uint4 *>(V_out + unit * cap_out * D);

    // Every load this phase needs is requested before the first result is used: V rows, norms and positions
    // of the rows stored ahead, the count of rows the two sets share, the query, the new row, the old scores
    // and norms (parked in LDS after the sweep, so that the later phases do not start with a round trip to
    // memory of their own), then the first 16 K rows of every thread.
    uint4 spec_k[kSpecSlots], spec_v[kSpecSlots];
    float spec_w[kSpecSlots];
    int spec_pos[kSpecSlots];
#pragma unroll
    for (int u = 0; u < kSpecSlots; ++u) {
        const int r = n - 1 - (u * kRowsPerPass + rloc);
        spec_v[u] = make_uint4(0, 0, 0, 0);
        spec_w[u] = 0.f;
        spec_pos[u] = 0;
        if (r >= spec_lo) {
            spec_v[u] = r == n0 ? vnew[sub] : load_rows<kStream>(Vu + static_cast<size_t>(r) * kLanesPerRow + sub);
            if (sub == 0 && r != n0) {
                spec_w[u] = Nu[r];
                if (pos) spec_pos[u] = pos[unit * cap + r];
            }
        }
    }
    const int synced = synced_in[unit];
    const uint4 q_raw = reinterpret_cast<const uint4 *>(q + unit * D)[sub];
    uint4 k_raw = make_uint4(0, 0, 0, 0);
    if (tid < kLanesPerRow) k_raw = knew[sub];
    float pre_s[kPre], pre_w[kPre];
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        const int r = tid + u * kOneThreads;
        pre_s[u] = r < n0 ? Su[r] : 0.f;
        pre_w[u] = r < n0 ? Nu[r] : 0.f;
    }

    // logits of all rows into LDS; the new row is read from the step's input, not from the cache
    for (int base = 0; base < n; base += kGroup * kRowsPerPass) {
        uint4 raw[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int r = n - 1 - (base + u * kRowsPerPass + rloc);
            const uint4 *src = (r == n0) ? knew + sub : Ku + static_cast<size_t>(r) * kLanesPerRow + sub;
            raw[u] = (r >= 0) ? load_rows<kStream>(src) : make_uint4(0, 0, 0, 0);
        }
        if (base == 0) {
            if (tid < kLanesPerRow) {
                // append the new row (slot 0 of these threads): k, v, |v|, pos
                reinterpret_cast<uint4 *>(K + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = k_raw;
                reinterpret_cast<uint4 *>(V + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = spec_v[0];
                const float new_norm = row_norm<T, kLanesPerRow>(norm, spec_v[0]);
                if (sub == 0) {
                    s_new_norm = new_norm;
                    Nu[n0] = new_norm;
                    if (pos) pos[unit * cap + n0] = len_pos.aux[b];
                    spec_w[0] = new_norm;
                    spec_pos[0] = len_pos.aux[b];
                }
            }
            // the rows behind the expected eviction go to the other set now, at the positions that guess implies
#pragma unroll
            for (int u = 0; u < kSpecSlots; ++u) {
                const int r = n - 1 - (u * kRowsPerPass + rloc);
                spec_k[u] = raw[u];
                if (r >= spec_lo && r != e_star) {
                    const int o = r - (r > e_star ? 1 : 0);
                    store_rows<kStream>(Ko + static_cast<size_t>(o) * kLanesPerRow + sub, raw[u]);
                    store_rows<kStream>(Vo + static_cast<size_t>(o) * kLanesPerRow + sub, spec_v[u]);
                    if (sub == 0) {
                        nrm_out[unit * cap_out + o] = spec_w[u];
                        if (pos_out) pos_out[unit * cap_out + o] = spec_pos[u];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int r = n - 1 - (base + u * kRowsPerPass + rloc);
            const float dot = group_all_reduce<kLanesPerRow>(dot_16_bytes<T>(raw[u], q_raw), OpSum{});
            if (sub == 0 && r >= 0) s_logit[r] = dot * scale_log2;
        }
    }
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        const int r = tid + u * kOneThreads;
        if (r < n0) { s_score[r] = pre_s[u]; s_norm[r] = pre_w[u]; }
    }
    // (a barrier for LDS only: the writes above must be visible, the V rows requested ahead need not have arrived)
    lds_barrier();
    if (tid == 0) { s_score[n0] = 0.f; s_norm[n0] = s_new_norm; }      // the appended row (published by the barriers below)

    // Statistics of every 128-row chunk, one wavefront per chunk and no exchange between wavefronts: the lane
    // takes rows lane and lane + 64 of the chunk -- the same function, on the same values, as in
    // decode_logits_kernel.
    const int n_chunks = (n + kDecodeChunk - 1) / kDecodeChunk;
    for (int chunk = wave; chunk < n_chunks; chunk += kWaves) {
        const int r0 = chunk * kDecodeChunk + lane, r1 = r0 + 64;
        const float2 st = chunk_stats_64x2(r0 < n ? s_logit[r0] : -INFINITY, r1 < n ? s_logit[r1] : -INFINITY);
        if (lane == 0) s_part[chunk] = st;
    }
    lds_barrier();
    float M, L;
    merge_chunk_stats(s_part, n_chunks, M, L);
    const float lse2 = M + log2f(L);

    auto new_score = [&](int r) { return s_score[r] + exp2f(s_logit[r] - lse2); };

    // the row that leaves: smallest importance among the unprotected rows, the highest row among equals.
    // A thread looks at rows tid, tid + 1024, ...: within a wavefront rows ascend with the lane, so the
    // wavefront's answer for one such round is the smallest key and the highest lane that holds it.
    int evicted = n;
    if (n > B) {
        unsigned long long best = ~0ull;
        for (int r0 = 0; r0 < n - recent; r0 += kOneThreads) {
            const int r = r0 + tid;
            const bool cand = r >= n_sink && r < n - recent;
            const unsigned key = cand ? __float_as_uint(__fmul_rn(new_score(r), s_norm[r])) : 0xffffffffu;
            const unsigned kmin = wave_min_u32(key);
            const unsigned long long holders = __ballot(cand && key == kmin);
            if (holders != 0ull) {
                const int top = 63 - __builtin_clzll(holders);
                const unsigned long long c = (static_cast<unsigned long long>(kmin) << 32) |
                                             static_cast<unsigned>(~static_cast<unsigned>(r0 + wave * 64 + top));
                best = c < best ? c : best;
            }
        }
        if (lane == 0) s_min[wave] = best;
        lds_barrier();
        best = s_min[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) best = s_min[w] < best ? s_min[w] : best;
        evicted = static_cast<int>(~static_cast<unsigned>(best & 0xffffffffull));
    }

    // rows of the other set that are out of date: from the first row in which it differs from the input
    // set, or from the evicted row if that comes earlier.  Source row r goes to row r - (r > evicted).
    const int first = min(synced, evicted);
    if (tid == 0) synced_out[unit] = evicted;

    // new scores and source rows of the survivors
    for (int o = tid; o < n_keep; o += kOneThreads) {
        const int src = o + (o >= evicted ? 1 : 0);
        if constexpr (kStream) {
            __builtin_nontemporal_store(new_score(src), &S_out[unit * cap_out + o]);
            if (kept_idx) __builtin_nontemporal_store(src, &kept_idx[unit * cap_out + o]);
        } else {
            S_out[unit * cap_out + o] = new_score(src);
            if (kept_idx) kept_idx[unit * cap_out + o] = src;
        }
    }

    // The rows from spec_lo on are in place already, except that a row e* which does not leave after all
    // (evicted < e*) has not been stored: it goes to e* - 1.
    if (evicted != e_star) {
#pragma unroll
        for (int u = 0; u < kSpecSlots; ++u) {
            const int r = n - 1 - (u * kRowsPerPass + rloc);
            if (r == e_star && r >= spec_lo) {
                const int o = r - 1;
                store_rows<kStream>(Ko + static_cast<size_t>(o) * kLanesPerRow + sub, spec_k[u]);
                store_rows<kStream>(Vo + static_cast<size_t>(o) * kLanesPerRow + sub, spec_v[u]);
                if (sub == 0) {
                    nrm_out[unit * cap_out + o] = spec_w[u];
                    if (pos_out) pos_out[unit * cap_out + o] = spec_pos[u];
                }
            }
        }
    }

    // ... and the rows before spec_lo that are out of date (the two sets were in step only up to a row
    // before it, or the evicted row lies before it) are copied from the cache as it was on entry: source
    // rows below spec_lo, never the appended row
    {
        const int o_end = min(n_keep, spec_lo - (evicted < spec_lo ? 1 : 0));
        for (int o = first + rloc; o < o_end; o += kRowsPerPass) {
            const int src = o + (o >= evicted ? 1 : 0);
            const uint4 kr = load_rows<kStream>(Ku + static_cast<size_t>(src) * kLanesPerRow + sub);
            const uint4 vr = load_rows<kStream>(Vu + static_cast<size_t>(src) * kLanesPerRow + sub);
            store_rows<kStream>(Ko + static_cast<size_t>(o) * kLanesPerRow + sub, kr);
            store_rows<kStream>(Vo + static_cast<size_t>(o) * kLanesPerRow + sub, vr);
            if (sub == 0) {
                nrm_out[unit * cap_out + o] = s_norm[src];
                if (pos_out) pos_out[unit * cap_out + o] = pos[unit * cap + src];
            }
        }
    }
}

}  // namespace

hipError_t launch_decode_prune(int dtype, int head_dim, const void *K, const void *V, const float *S,
                               const float *nrm, const int32_t *pos, void *K_out, void *V_out, float *S_out,
                               float *nrm_out, int32_t *pos_out, int32_t *kept_idx, const int32_t *synced_in,
                               int32_t *synced_out, const float *ws_logit, const float2 *ws_part,
                               const float *ws_out, float *out, const WindowArgs &win, const BatchMeta &meta,
                               const Geometry &g, hipStream_t st)
{
    const int chunks_alloc = (g.cap + kDecodeChunk - 1) / kDecodeChunk;
    const unsigned units = static_cast<unsigned>(g.batch) * g.n_heads;
    // Workgroups per head: each of them repeats the scan over all of the head's rows (group times as many logits
    // with grouped queries), so more of them only pay while the chip is not yet full.  Measured per step: 512 heads
    // (ragged16) 49.8 us with one, 51.2 with two, 56 with four; 64 heads x 4 query heads 28 us with 2 to 8, 35 with 16.
    unsigned G = 512u / (units * static_cast<unsigned>(g.group));
    G = G < 1u ? 1u : (G > 16u ? 16u : G);
    dim3 grid(units, G), block(kThreads);
#define VATP_DPG(T, D, G)                                                                                      \
    hipLaunchKernelGGL((decode_prune_kernel<T, D, G>), grid, block, 0, st, static_cast<const T *>(K),            \
                       static_cast<const T *>(V), S, nrm, pos, static_cast<T *>(K_out), static_cast<T *>(V_out), \
                       S_out, nrm_out, pos_out, kept_idx, synced_in, synced_out, ws_logit, ws_part, ws_out, out, \
                       win, meta, g.n_heads, g.cap, g.cap_out, chunks_alloc, g.n_sink, g.recent, g.group, g.stream)
    // (instantiated for group sizes up to 2, 4, 8 and 16: the smallest that fits)
#define VATP_DP(T, D)                                      \
    do {                                                   \
        if (g.group > 8) VATP_DPG(T, D, VATP_MAX_GROUP);   \
        else if (g.group > 4) VATP_DPG(T, D, 8);           \
        else if (g.group > 2) VATP_DPG(T, D, 4);           \
        else if (g.group > 1) VATP_DPG(T, D, 2);           \
        else VATP_DPG(T, D, 1);                            \
    } while (0)
    if (dtype == VATP_F32 && head_dim == 64) VATP_DP(float, 64);
    else if (dtype == VATP_F32) VATP_DP(float, 128);
    else if (head_dim == 64) VATP_DP(bf16_t, 64);
    else VATP_DP(bf16_t, 128);
#undef VATP_DP
#undef VATP_DPG
    return hipGetLastError();
}

}  // namespace vatp

namespace vatp {

int decode_prune_one_max_rows() { return kOneMaxRows; }

hipError_t launch_decode_prune_one(int dtype, int head_dim, const void *q, const void *k, const void *v, void *K,
                                   void *V, const float *S, float *nrm, int32_t *pos, void *K_out, void *V_out,
                                   float *S_out, float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                                   const int32_t *synced_in, int32_t *synced_out, const BatchMeta &len_pos,
                                   const BudgetList &budget, const Geometry &g, hipStream_t st)
{
    const unsigned units = static_cast<unsigned>(g.batch) * g.n_heads;
    dim3 grid(units), block(kOneThreads);
#define VATP_DP1(T, D)                                                                                           \
    do {                                                                                                         \
        if (g.stream) VATP_DP1_S(T, D, true);                                                                    \
        else VATP_DP1_S(T, D, false);                                                                            \
    } while (0)
#define VATP_DP1_S(T, D, STREAM)                                                                                    \
    hipLaunchKernelGGL((decode_prune_one_kernel<T, D, STREAM>), grid, block, 0, st, static_cast<const T *>(q),         \
                       static_cast<const T *>(k), static_cast<const T *>(v), static_cast<T *>(K),                \
                       static_cast<T *>(V), S, nrm, pos, static_cast<T *>(K_out), static_cast<T *>(V_out), S_out, \
                       nrm_out, pos_out, kept_idx, synced_in, synced_out, len_pos, budget, g.n_heads, g.cap,     \
                       g.cap_out, g.n_sink, g.recent, g.scale_log2, g.norm)
    if (dtype == VATP_F32 && head_dim == 64) VATP_DP1(float, 64);
    else if (dtype == VATP_F32) VATP_DP1(float, 128);
    else if (head_dim == 64) VATP_DP1(bf16_t, 64);
    else VATP_DP1(bf16_t, 128);
#undef VATP_DP1
#undef VATP_DP1_S
    return hipGetLastError();
}

}  // namespace vatp
