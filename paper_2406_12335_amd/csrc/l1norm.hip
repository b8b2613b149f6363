// Norm of every value row (paper Eq. 4: l1; Table 2 ablation: l2, l-infinity), HBM-bound.
// A row of head_dim elements is read by a group of lanes, 16 bytes per lane, so that a
// wavefront's load covers consecutive rows as one contiguous span.
#include "vatp_device.h"

namespace vatp {

template <typename T, int D>
__global__ __launch_bounds__(256) void l1norm_kernel(const T *__restrict__ V,
                                                     float *__restrict__ nrm, BatchMeta meta,
                                                     int n_heads, int cap, int norm)
{
    constexpr int kE = Elt<T>::kPer16B;          // elements per 16-byte lane load
    constexpr int kLanesPerRow = D / kE;         // 8, 16 or 32
    constexpr int kRowsPerPass = 256 / kLanesPerRow;
    constexpr int kRowsPerBlock = 256;

    const int b = blockIdx.z, h = blockIdx.y;
    const int len = meta.len[b];
    const int row0 = blockIdx.x * kRowsPerBlock;
    if (row0 >= len) return;
    const size_t unit = static_cast<size_t>(b) * n_heads + h;
    const uint4 *Vu = reinterpret_cast<const uint4 *>(V + unit * cap * D);
    float *nu = nrm + unit * cap;

    const int sub = threadIdx.x % kLanesPerRow;
    const int rloc = threadIdx.x / kLanesPerRow;
    // all of the workgroup's row loads are issued before the first one is used
    constexpr int kPasses = kRowsPerBlock / kRowsPerPass;
    constexpr int kGroup = kPasses < 16 ? kPasses : 16;
#pragma unroll
    for (int p0 = 0; p0 < kPasses; p0 += kGroup) {
        uint4 raw[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int r = row0 + (p0 + u) * kRowsPerPass + rloc;
            raw[u] = r < len ? Vu[static_cast<size_t>(r) * kLanesPerRow + sub] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int r = row0 + (p0 + u) * kRowsPerPass + rloc;
            const float value = row_norm<T, kLanesPerRow>(norm, raw[u]);
            if (sub == 0 && r < len) nu[r] = value;
        }
    }
}

hipError_t launch_l1norm(int dtype, int head_dim, const void *V, float *nrm,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st)
{
    if (g.max_len <= 0) return hipSuccess;
    dim3 grid((g.max_len + 255) / 256, g.n_heads, g.batch), block(256);
#define VATP_L1(T, D)                                                                        \
    hipLaunchKernelGGL((l1norm_kernel<T, D>), grid, block, 0, st, static_cast<const T *>(V), \
                       nrm, meta, g.n_heads, g.cap, g.norm)
    if (dtype == VATP_F32 && head_dim == 64) VATP_L1(float, 64);
    else if (dtype == VATP_F32) VATP_L1(float, 128);
    else if (head_dim == 64) VATP_L1(bf16_t, 64);
    else VATP_L1(bf16_t, 128);
#undef VATP_L1
    return hipGetLastError();
}

}  // namespace vatp
