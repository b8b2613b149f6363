// Internal declarations shared by the HIP sources of libvatp (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vatp.h"

namespace vatp {

typedef uint16_t bf16_t;   // raw bfloat16 bits

// Per-sequence host facts, passed to kernels by value (lives in the kernarg segment,
// read with scalar loads indexed by blockIdx.z): no device copy, no sync.
struct BatchMeta {
    int32_t len[VATP_MAX_BATCH];   // rows valid per sequence on entry
    int32_t aux[VATP_MAX_BATCH];   // budget (select/compact) or new_pos (decode)
};

struct Geometry {
    int32_t batch, n_heads, cap, cap_out;
    int32_t n_sink, recent;
    float   scale_log2;            // c * log2(e): logits are kept in the base-2 domain
    int32_t max_len;               // max over the batch of len (decode: len + 1)
    int32_t norm;                  // VATP_NORM_*: value-row norm of the importance (paper Eq. 4, Table 2)
};

// Value-row norm in three steps: lane-local accumulation, combination across the row's lanes,
// final map.  l1 (the paper's metric), l2 and l-infinity (its ablation, Table 2).
__device__ __forceinline__ float norm_accum(int kind, float acc, float x) {
    return kind == VATP_NORM_L1 ? acc + fabsf(x) : kind == VATP_NORM_L2 ? fmaf(x, x, acc) : fmaxf(acc, fabsf(x));
}
__device__ __forceinline__ float norm_combine(int kind, float a, float b) {
    return kind == VATP_NORM_LINF ? fmaxf(a, b) : a + b;
}
__device__ __forceinline__ float norm_finish(int kind, float a) { return kind == VATP_NORM_L2 ? sqrtf(a) : a; }

constexpr int kDecodeChunk = 128;  // rows of one unit handled by one workgroup of the decode GEMV

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
    return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

template <typename T> struct Elt;
template <> struct Elt<float> {
    static constexpr int kPer16B = 4;
    __device__ static __forceinline__ void unpack(const uint4 &raw, float *out) {
        out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
        out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
    }
};
template <> struct Elt<bf16_t> {
    static constexpr int kPer16B = 8;
    __device__ static __forceinline__ void unpack(const uint4 &raw, float *out) {
        out[0] = __uint_as_float(raw.x << 16); out[1] = __uint_as_float(raw.x & 0xffff0000u);
        out[2] = __uint_as_float(raw.y << 16); out[3] = __uint_as_float(raw.y & 0xffff0000u);
        out[4] = __uint_as_float(raw.z << 16); out[5] = __uint_as_float(raw.z & 0xffff0000u);
        out[6] = __uint_as_float(raw.w << 16); out[7] = __uint_as_float(raw.w & 0xffff0000u);
    }
};

// ---- host-side launchers, one per source file --------------------------------------
hipError_t launch_l1norm(int dtype, int head_dim, const void *V, float *nrm,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

hipError_t launch_prefill_generic(int dtype, int head_dim, const void *Q, const void *K,
                                  float *S, float *lse2, bool have_lse, const BatchMeta &meta,
                                  const Geometry &g, hipStream_t st);

hipError_t launch_lse_to_base2(const float *lse, float *lse2, const BatchMeta &meta, const Geometry &g,
                               hipStream_t st);

hipError_t launch_prefill_mfma(const void *Q, const void *K, float *S, float *lse2, bool have_lse,
                               const BatchMeta &meta, const Geometry &g, hipStream_t st);

hipError_t launch_decode(int dtype, int head_dim, const void *q, const void *k, const void *v,
                         void *K, void *V, float *S, float *nrm, int32_t *pos,
                         float *ws_logit, float2 *ws_part, float *ws_out, float *out, const BatchMeta &meta,
                         const Geometry &g, hipStream_t st);

hipError_t launch_select(const float *S, const float *nrm, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

hipError_t launch_gather(int dtype, int head_dim, bool evict_one,
                         const void *K, const void *V, const float *S, const float *nrm,
                         const int32_t *pos, void *K_out, void *V_out, float *S_out,
                         float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                         const BatchMeta &meta, const Geometry &g, hipStream_t st);

}  // namespace vatp
