// One decode step of the accumulated attention score (paper Eq. 2, taken incrementally;
// order of operations as in Fig. 2): append the new token's row, let its query attend
// over every cached row, add the attention weights to the rows' running scores.
//
// Two launches, no atomics, no fences:
//   logits  HBM-bound GEMV.  A (batch, head) unit is cut into chunks of kDecodeChunk rows, one
//           workgroup each, so that even a single sequence fills the chip.  Every K row is
//           read exactly once, 16 bytes per lane, a group of lanes per row, all of the
//           workgroup's loads in flight before the first is used.  The workgroup leaves its
//           logits (base-2 domain, t = c*log2(e)*<q,k>) and its chunk's (max, sum of 2^(t-max))
//           in the workspace, and the one that owns the new row appends k, v, |v|_1 and pos.
//           With an output pointer (vatp_decode_attend_step) it also reads the V rows and leaves
//           the chunk's unnormalised share of the attention output (Eq. 1) in the workspace.
//   finish  one row per thread: every wavefront merges the unit's few chunk statistics into
//           log2 sum 2^t and applies S += 2^(t - lse2); 12 bytes per row, a tiny launch
//           ordered after the first by the stream.
#include "vatp_device.h"

namespace vatp {

namespace {

template <typename T, int D, bool kAttend, bool kStream>
__global__ __launch_bounds__(256) void decode_logits_kernel(
    const T *__restrict__ q, const T *__restrict__ k_new, const T *__restrict__ v_new,
    T *__restrict__ K, T *__restrict__ V, float *__restrict__ nrm, int32_t *__restrict__ pos,
    float *__restrict__ ws_logit, float2 *__restrict__ ws_part, float *__restrict__ ws_out,
    BatchMeta meta, int n_heads, int cap, int chunks_alloc, float scale_log2, int norm)
{
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = 256 / kLanesPerRow;
    constexpr int kPasses = kDecodeChunk / kRowsPerPass;
    constexpr int kGroup = kPasses < 16 ? kPasses : 16;        // loads issued back to back

    __shared__ float s_logit[kDecodeChunk];

    // unit in the fast grid dimension: workgroups go to the 8 XCDs round-robin by linear id, so (with a
    // unit count that is a multiple of 8) a head's chunks, and the launch that consumes their logits,
    // share one XCD's L2
    const size_t unit = blockIdx.x;
    const int b = static_cast<int>(unit / n_heads), chunk = blockIdx.y;
    const int n0 = meta.len[b];            // rows cached before this step = index of the new row
    const int n = n0 + 1;
    const int row0 = chunk * kDecodeChunk;
    if (row0 >= n) return;
    const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
    const uint4 *knew = reinterpret_cast<const uint4 *>(k_new + unit * D);
    const int tid = threadIdx.x;
    const int sub = tid % kLanesPerRow;
    const int rloc = tid / kLanesPerRow;
    const int lane = tid & 63, wave = tid >> 6;

    // Every load of this phase is requested before the first result is used: the query, the new row (in the
    // workgroup that owns it), then all of the workgroup's K rows.
    const uint4 q_raw = reinterpret_cast<const uint4 *>(q + unit * D)[sub];
    const bool owns_new_row = n0 >= row0 && n0 < row0 + kDecodeChunk && tid < kLanesPerRow;
    uint4 kraw = make_uint4(0, 0, 0, 0), vraw = make_uint4(0, 0, 0, 0);
    if (owns_new_row) {
        kraw = knew[sub];
        vraw = reinterpret_cast<const uint4 *>(v_new + unit * D)[sub];
    }

    // logits of the chunk's rows; the new row is read from the step's input, not from the cache
#pragma unroll
    for (int p0 = 0; p0 < kPasses; p0 += kGroup) {
        uint4 raw[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int r = row0 + (p0 + u) * kRowsPerPass + rloc;
            const uint4 *src = (r == n0) ? knew + sub : Ku + static_cast<size_t>(r) * kLanesPerRow + sub;
            raw[u] = (r < n) ? load_rows<kStream>(src) : make_uint4(0, 0, 0, 0);
        }
        if (p0 == 0 && owns_new_row) {
            // the workgroup that owns the new row stores k, v, |v| and pos into the caches
            reinterpret_cast<uint4 *>(K + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = kraw;
            reinterpret_cast<uint4 *>(V + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = vraw;
            const float new_norm = row_norm<T, kLanesPerRow>(norm, vraw);
            if (sub == 0) {
                nrm[unit * cap + n0] = new_norm;
                if (pos) pos[unit * cap + n0] = meta.aux[b];
            }
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int rl = (p0 + u) * kRowsPerPass + rloc;
            const float dot = group_all_reduce<kLanesPerRow>(dot_16_bytes<T>(raw[u], q_raw), OpSum{});
            if (sub == 0) s_logit[rl] = (row0 + rl < n) ? dot * scale_log2 : -INFINITY;
        }
    }
    __syncthreads();

    // the chunk's logits go to the workspace; its statistics (maximum, sum of 2^(t - max)) are formed by one
    // wavefront, two rows per lane, without any exchange between wavefronts
    if (tid < kDecodeChunk && row0 + tid < n) ws_logit[unit * cap + row0 + tid] = s_logit[tid];
    float2 st = make_float2(0.f, 0.f);
    if (wave == 0 || kAttend) {
        st = chunk_stats_64x2(s_logit[lane], s_logit[lane + 64]);
        if (tid == 0) ws_part[unit * chunks_alloc + chunk] = st;
    }

    if constexpr (kAttend) {
        // this chunk's share of the attention output (paper Eq. 1), unnormalised and relative to the
        // chunk maximum:  o_c = sum_r 2^(t_r - max_c) v_r ; the finish launch rescales and adds the chunks
        // (every wavefront has formed the chunk maximum for itself above)
        const float mx = st.x;
        __shared__ float s_o[kRowsPerPass][D];
        const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * D);
        const uint4 *vnew = reinterpret_cast<const uint4 *>(v_new + unit * D);
        float oacc[kE];
#pragma unroll
        for (int e = 0; e < kE; ++e) oacc[e] = 0.f;
#pragma unroll
        for (int p0 = 0; p0 < kPasses; p0 += kGroup) {
            uint4 raw[kGroup];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int r = row0 + (p0 + u) * kRowsPerPass + rloc;
                const uint4 *src = (r == n0) ? vnew + sub : Vu + static_cast<size_t>(r) * kLanesPerRow + sub;
                raw[u] = (r < n) ? load_rows<kStream>(src) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const float p = exp2f(s_logit[(p0 + u) * kRowsPerPass + rloc] - mx);   // 0 past the end
                float vf[kE];
                Elt<T>::unpack(raw[u], vf);
#pragma unroll
                for (int e = 0; e < kE; ++e) oacc[e] = fmaf(p, vf[e], oacc[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < kE; ++e) s_o[rloc][sub * kE + e] = oacc[e];
        __syncthreads();
        if (tid < D) {
            float o = 0.f;
#pragma unroll
            for (int g = 0; g < kRowsPerPass; ++g) o += s_o[g][tid];
            ws_out[(unit * chunks_alloc + chunk) * D + tid] = o;
        }
    }
}

// The same launch for grouped-query attention: the workgroup reads its chunk of K rows once and
// forms the logits of all g query heads of the group against it (the point of sharing a K/V head:
// the cache is read once per group, not once per query head).  Logits and chunk statistics are kept
// per query head ([g, cap] and [g, chunks] per unit); with an output pointer each head's share of
// its attention output as well.
template <typename T, int D, bool kAttend, bool kStream>
__global__ __launch_bounds__(256) void decode_logits_group_kernel(
    const T *__restrict__ q, const T *__restrict__ k_new, const T *__restrict__ v_new,
    T *__restrict__ K, T *__restrict__ V, float *__restrict__ nrm, int32_t *__restrict__ pos,
    float *__restrict__ ws_logit, float2 *__restrict__ ws_part, float *__restrict__ ws_out,
    BatchMeta meta, int n_heads, int cap, int chunks_alloc, float scale_log2, int norm, int group)
{
    constexpr int kG = VATP_MAX_GROUP;
    constexpr int kE = Elt<T>::kPer16B;
    constexpr int kLanesPerRow = D / kE;
    constexpr int kRowsPerPass = 256 / kLanesPerRow;
    constexpr int kPasses = kDecodeChunk / kRowsPerPass;
    constexpr int kGroup = kPasses;                            // all of a thread's row loads are issued back to back
    static_assert(kGroup == kLanesPerRow / 2 && kGroup <= 16, "the butterfly below pairs rows with lanes");

    __shared__ float s_logit[kG][kDecodeChunk];
    __shared__ float s_max[kG];

    const size_t unit = blockIdx.x;                            // K/V head
    const int b = static_cast<int>(unit / n_heads), chunk = blockIdx.y;
    const int n0 = meta.len[b];
    const int n = n0 + 1;
    const int row0 = chunk * kDecodeChunk;
    if (row0 >= n) return;
    const uint4 *Ku = reinterpret_cast<const uint4 *>(K + unit * cap * D);
    const uint4 *knew = reinterpret_cast<const uint4 *>(k_new + unit * D);
    const int tid = threadIdx.x;
    const int sub = tid % kLanesPerRow;
    const int rloc = tid / kLanesPerRow;
    const int lane = tid & 63, wave = tid >> 6;

    // bf16 rows of 128 elements: the logits of a group are a (rows x 128) by (128 x g) product and go to the
    // matrix cores (the chunk's rows staged in LDS, every wavefront one 32-row tile); other shapes use FMAs
    constexpr bool kMfma = sizeof(T) == 2 && D == 128;
    constexpr int kQ = kMfma ? 8 : kG;      // per lane: 8 MFMA steps' worth of one head, or a slice of every head
    uint4 q_raw[kQ];
#pragma unroll
    for (int i = 0; i < kQ; ++i) {
        q_raw[i] = make_uint4(0, 0, 0, 0);
        if constexpr (kMfma) {
            // B operand of MFMA step i: this lane's 8 elements of query head lane & 31 (zero beyond the group)
            if ((lane & 31) < group)
                q_raw[i] = reinterpret_cast<const uint4 *>(q + (unit * group + (lane & 31)) * D)[i + 8 * (lane >> 5)];
        } else {
            if (i < group) q_raw[i] = reinterpret_cast<const uint4 *>(q + (unit * group + i) * D)[sub];
        }
    }
    const bool owns_new_row = n0 >= row0 && n0 < row0 + kDecodeChunk && tid < kLanesPerRow;
    uint4 kraw = make_uint4(0, 0, 0, 0), vraw = make_uint4(0, 0, 0, 0);
    if (owns_new_row) {
        kraw = knew[sub];
        vraw = reinterpret_cast<const uint4 *>(v_new + unit * D)[sub];
    }
    float qf[kG][kE];

#pragma unroll
    for (int p0 = 0; p0 < kPasses; p0 += kGroup) {
        uint4 raw[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int r = row0 + (p0 + u) * kRowsPerPass + rloc;
            const uint4 *src = (r == n0) ? knew + sub : Ku + static_cast<size_t>(r) * kLanesPerRow + sub;
            raw[u] = (r < n) ? load_rows<kStream>(src) : make_uint4(0, 0, 0, 0);
        }
        if (p0 == 0) {
            if constexpr (!kMfma) {
#pragma unroll
                for (int i = 0; i < kG; ++i) Elt<T>::unpack(q_raw[i], qf[i]);
            }
            if (owns_new_row) {                     // append k, v, |v| and pos
                reinterpret_cast<uint4 *>(K + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = kraw;
                reinterpret_cast<uint4 *>(V + unit * cap * D)[static_cast<size_t>(n0) * kLanesPerRow + sub] = vraw;
                const float new_norm = row_norm<T, kLanesPerRow>(norm, vraw);
                if (sub == 0) {
                    nrm[unit * cap + n0] = new_norm;
                    if (pos) pos[unit * cap + n0] = meta.aux[b];
                }
            }
        }
        if constexpr (kMfma) {
            static_assert(!kMfma || (kG <= 32 && kGroup == 8 && kLanesPerRow == 16), "8 MFMA steps of 16 over the 128 elements, a head per column");
            __shared__ uint4 s_k[kDecodeChunk * kLanesPerRow];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int rl = u * kRowsPerPass + rloc;
                s_k[rl * kLanesPerRow + swizzled_chunk(rl, sub)] = raw[u];
            }
            __syncthreads();
            const int ln = lane & 31, gl = lane >> 5;
            const int ar = 32 * wave + ln;             // this lane's row of the wavefront's tile
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int st = 0; st < 8; ++st)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    as_bf16x8(s_k[ar * kLanesPerRow + swizzled_chunk(ar, st + 8 * gl)]), as_bf16x8(q_raw[st]), acc, 0, 0, 0);
            if (ln < group) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = 32 * wave + acc_row(v) + 4 * gl;
                    s_logit[ln][rl] = (row0 + rl < n) ? acc[v] * scale_log2 : -INFINITY;
                }
            }
        } else {
            float kf[kGroup][kE];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) Elt<T>::unpack(raw[u], kf[u]);
#pragma unroll
            for (int i = 0; i < kG; ++i) {
                if (i >= group) continue;
                // this lane's share of the dot products of head i with its kGroup rows ...
                float part[kGroup];
#pragma unroll
                for (int u = 0; u < kGroup; ++u) {
                    part[u] = 0.f;
#pragma unroll
                    for (int e = 0; e < kE; ++e) part[u] = fmaf(qf[i][e], kf[u][e], part[u]);
                }
                // ... summed over the row's lanes by a butterfly that halves the number of rows a lane is
                // responsible for at every step (the lane with the offset bit set keeps the upper half and
                // hands over the lower one): kGroup - 1 exchanges instead of kGroup * log2(lanes per row).
                // The lane ends up with the whole sum of row sub / 2.
#pragma unroll
                for (int off = kLanesPerRow / 2; off >= 2; off >>= 1) {
                    const int half = off / 2;
                    const bool upper = (sub & off) != 0;
#pragma unroll
                    for (int j = 0; j < half; ++j) {
                        const float send = upper ? part[j] : part[j + half];
                        const float keep = upper ? part[j + half] : part[j];
                        part[j] = keep + __shfl_xor(send, off);
                    }
                }
                part[0] += __shfl_xor(part[0], 1);
                if ((sub & 1) == 0) {
                    const int rl = (p0 + (sub >> 1)) * kRowsPerPass + rloc;
                    s_logit[i][rl] = (row0 + rl < n) ? part[0] * scale_log2 : -INFINITY;
                }
            }
        }
    }
    __syncthreads();

    // chunk statistics, one wavefront per query head (two rows per lane): no exchange between wavefronts
    for (int i = wave; i < group; i += 4) {
        const float2 st = chunk_stats_64x2(s_logit[i][lane], s_logit[i][lane + 64]);
        if (lane == 0) {
            ws_part[(unit * group + i) * chunks_alloc + chunk] = st;
            s_max[i] = st.x;
        }
    }
    for (int idx = tid; idx < group * kDecodeChunk; idx += 256) {
        const int i = idx / kDecodeChunk, r = idx % kDecodeChunk;
        if (row0 + r < n) ws_logit[(unit * group + i) * cap + row0 + r] = s_logit[i][r];
    }

    if constexpr (kAttend) {
        // every head's share of its attention output (Eq. 1) over this chunk, relative to the head's
        // chunk maximum; rows are summed inside the wavefront first, then across the four through LDS
        __shared__ float s_o[4][kG][D];
        __syncthreads();                                      // s_max
        const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * D);
        const uint4 *vnew = reinterpret_cast<const uint4 *>(v_new + unit * D);
        float oacc[kG][kE];
#pragma unroll
        for (int i = 0; i < kG; ++i)
#pragma unroll
            for (int e = 0; e < kE; ++e) oacc[i][e] = 0.f;
#pragma unroll
        for (int p0 = 0; p0 < kPasses; p0 += kGroup) {
            uint4 raw[kGroup];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int r = row0 + (p0 + u) * kRowsPerPass + rloc;
                const uint4 *src = (r == n0) ? vnew + sub : Vu + static_cast<size_t>(r) * kLanesPerRow + sub;
                raw[u] = (r < n) ? load_rows<kStream>(src) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int rl = (p0 + u) * kRowsPerPass + rloc;
                float vf[kE];
                Elt<T>::unpack(raw[u], vf);
#pragma unroll
                for (int i = 0; i < kG; ++i) {
                    if (i >= group) continue;
                    const float p = exp2f(s_logit[i][rl] - s_max[i]);       // 0 past the end
#pragma unroll
                    for (int e = 0; e < kE; ++e) oacc[i][e] = fmaf(p, vf[e], oacc[i][e]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kG; ++i) {
            if (i >= group) continue;
#pragma unroll
            for (int e = 0; e < kE; ++e) {
                float o = oacc[i][e];
#pragma unroll
                for (int off = kLanesPerRow; off < 64; off <<= 1) o += __shfl_xor(o, off);
                if (lane < kLanesPerRow) s_o[wave][i][sub * kE + e] = o;
            }
        }
        __syncthreads();
        for (int idx = tid; idx < group * D; idx += 256) {
            const int i = idx / D, x = idx % D;
            ws_out[((unit * group + i) * chunks_alloc + chunk) * D + x] =
                (s_o[0][i][x] + s_o[1][i][x]) + (s_o[2][i][x] + s_o[3][i][x]);
        }
    }
}

template <int kMaxG>
__global__ __launch_bounds__(256) void decode_finish_kernel(float *__restrict__ S,
                                                            const float *__restrict__ ws_logit,
                                                            const float2 *__restrict__ ws_part,
                                                            const float *__restrict__ ws_out,
                                                            float *__restrict__ out, int head_dim,
                                                            BatchMeta meta, int n_heads, int cap,
                                                            int chunks_alloc, int group)
{
    const size_t unit = blockIdx.x;
    const int b = static_cast<int>(unit / n_heads);
    const int n0 = meta.len[b], n = n0 + 1;
    const int row0 = static_cast<int>(blockIdx.y) * 256;
    const int r = row0 + static_cast<int>(threadIdx.x);          // one row per thread
    if (row0 >= n) return;
    float logit[kMaxG], s_old = 0.f;
    load_group_logits<kMaxG>(logit, ws_logit + unit * group * cap, cap, group, r, r < n);
    if (r < n && r != n0) s_old = S[unit * cap + r];
    // the softmax denominators from the unit's chunk statistics (per wavefront, one round trip)
    const int n_chunks = (n + kDecodeChunk - 1) / kDecodeChunk;
    const float2 *part = ws_part + unit * group * chunks_alloc;
    float lse2[kMaxG];
    merge_group_stats<kMaxG>(part, chunks_alloc, group, n_chunks, lse2);
    if (r < n) S[unit * cap + r] = s_old + group_weight<kMaxG>(logit, lse2, group);
    // attention output of the new token, per query head: the chunks' partial sums, rescaled to the common maximum
    if (out && blockIdx.y == 0)
        merge_group_outputs(out + unit * group * head_dim, ws_out + unit * group * chunks_alloc * head_dim, part, chunks_alloc,
                            n_chunks, group, head_dim, 256);
}

}  // namespace

hipError_t launch_decode(int dtype, int head_dim, const void *q, const void *k, const void *v,
                         void *K, void *V, float *S, float *nrm, int32_t *pos, float *ws_logit,
                         float2 *ws_part, float *ws_out, float *out, bool finish, const BatchMeta &meta,
                         const Geometry &g, hipStream_t st)
{
    const int chunks_alloc = (g.cap + kDecodeChunk - 1) / kDecodeChunk;
    const unsigned units = static_cast<unsigned>(g.batch) * g.n_heads;
    dim3 grid(units, (g.max_len + kDecodeChunk - 1) / kDecodeChunk), block(256);
    const bool attend = ws_out != nullptr;
#define VATP_DEC_S(KERNEL, T, D, A, STREAM, ...)                                                           \
    hipLaunchKernelGGL((KERNEL<T, D, A, STREAM>), grid, block, 0, st, static_cast<const T *>(q),            \
                       static_cast<const T *>(k), static_cast<const T *>(v), static_cast<T *>(K),      \
                       static_cast<T *>(V), nrm, pos, ws_logit, ws_part, ws_out, meta, g.n_heads,      \
                       g.cap, chunks_alloc, g.scale_log2, g.norm, ##__VA_ARGS__)
#define VATP_DEC(KERNEL, T, D, A, ...)                                                                 \
    do {                                                                                               \
        if (g.stream) VATP_DEC_S(KERNEL, T, D, A, true, ##__VA_ARGS__);                                \
        else VATP_DEC_S(KERNEL, T, D, A, false, ##__VA_ARGS__);                                        \
    } while (0)
#define VATP_DEC2(T, D)                                                                                \
    do {                                                                                               \
        if (g.group > 1) {                                                                             \
            if (attend) VATP_DEC(decode_logits_group_kernel, T, D, true, g.group);                     \
            else VATP_DEC(decode_logits_group_kernel, T, D, false, g.group);                           \
        } else {                                                                                       \
            if (attend) VATP_DEC(decode_logits_kernel, T, D, true);                                    \
            else VATP_DEC(decode_logits_kernel, T, D, false);                                          \
        }                                                                                              \
    } while (0)
    if (dtype == VATP_F32 && head_dim == 64) VATP_DEC2(float, 64);
    else if (dtype == VATP_F32) VATP_DEC2(float, 128);
    else if (head_dim == 64) VATP_DEC2(bf16_t, 64);
    else VATP_DEC2(bf16_t, 128);
#undef VATP_DEC2
#undef VATP_DEC
#undef VATP_DEC_S
    if (finish) {   // (the fused decode-and-evict step has its own second launch)
        const dim3 fgrid(units, (g.max_len + 255) / 256);
#define VATP_FIN(G)                                                                                               \
    hipLaunchKernelGGL(decode_finish_kernel<G>, fgrid, block, 0, st, S, ws_logit, ws_part, ws_out, out, head_dim, meta, \
                       g.n_heads, g.cap, chunks_alloc, g.group)
        if (g.group > 8) VATP_FIN(VATP_MAX_GROUP);
        else if (g.group > 4) VATP_FIN(8);
        else if (g.group > 2) VATP_FIN(4);
        else if (g.group > 1) VATP_FIN(2);
        else VATP_FIN(1);
#undef VATP_FIN
    }
    return hipGetLastError();
}

}  // namespace vatp
