// Causal attention, one wave per (query row, query head): the form used by the token-by-token decode path
// (one query against its KV cache) and by the fp32 model path.  Keys are walked 64 at a time (one key per
// lane for the scores, one or more channels per lane for the weighted value sum) with an online softmax in
// fp32.  The bf16 prefill uses the matrix-core kernel in kernels_attn_mfma.hip instead.
#include "common.h"
#include "kernels.h"

namespace vl {

template <typename T> __device__ __forceinline__ void load4(const T* p, float (&v)[4]);
template <> __device__ __forceinline__ void load4<float>(const float* p, float (&v)[4]) {
    const float4 t = *(const float4*)p;
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ __forceinline__ void load4<bf16>(const bf16* p, float (&v)[4]) {
    const bf16x4 t = *(const bf16x4*)p;
    v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
}

template <typename T>
__global__ __launch_bounds__(64) void attn_rowwise_kernel(const T* __restrict__ q, int64_t q_stride,
                                                          const T* __restrict__ k, const T* __restrict__ v,
                                                          int64_t kv_stride, const int32_t* __restrict__ kv_row0,
                                                          const int32_t* __restrict__ npos, T* __restrict__ out,
                                                          int hq, int hkv, int hd, float scale, bool out_tiled) {
    __shared__ float qs[256];
    const int64_t row = blockIdx.x;
    const int j = blockIdx.y, g = j / (hq / hkv), lane = threadIdx.x;
    const int nkeys = npos[row] + 1;
    const int64_t base = (int64_t)kv_row0[row];
    for (int c = lane; c < hd; c += WAVE) qs[c] = to_f32(q[row * q_stride + (int64_t)j * hd + c]);
    __syncthreads();
    float m = -INFINITY, l = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < nkeys; t0 += WAVE) {
        const int t = t0 + lane;
        float sc = -INFINITY;
        if (t < nkeys) {
            const T* kp = k + (base + t) * kv_stride + (int64_t)g * hd;
            float dot = 0.f;
            for (int c = 0; c < hd; c += 4) {
                float kv4[4];
                load4<T>(kp + c, kv4);
                dot = fmaf(qs[c], kv4[0], dot);
                dot = fmaf(qs[c + 1], kv4[1], dot);
                dot = fmaf(qs[c + 2], kv4[2], dot);
                dot = fmaf(qs[c + 3], kv4[3], dot);
            }
            sc = dot * scale;
        }
        const float mnew = fmaxf(m, wave_max(sc));
        const float p = (t < nkeys) ? expf(sc - mnew) : 0.f;
        const float corr = expf(m - mnew);
        l = l * corr + wave_sum(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] *= corr;
        const int cnt = min(WAVE, nkeys - t0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, WAVE);
            const T* vp = v + (base + t0 + jj) * kv_stride + (int64_t)g * hd;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = lane + WAVE * i;
                if (c < hd) o[i] = fmaf(pj, to_f32(vp[c]), o[i]);
            }
        }
        m = mnew;
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + WAVE * i;
        if (c < hd) out[out_tiled ? tiled_off(row, j * hd + c, (int64_t)hq * hd) : row * (int64_t)hq * hd + (int64_t)j * hd + c] = from_f32<T>(o[i] * inv);
    }
}

void launch_attn_rowwise(const void* q, int64_t q_stride, const void* k, const void* v, int64_t kv_stride,
                         const int32_t* kv_row0, const int32_t* npos, void* out, int dtype, int64_t rows, int hq,
                         int hkv, int hd, hipStream_t s, bool out_tiled) {
    if (rows <= 0) return;
    const float scale = 1.0f / sqrtf((float)hd);
    dim3 grid((unsigned)rows, (unsigned)hq);
    if (dtype == VL_BF16)
        attn_rowwise_kernel<bf16><<<grid, 64, 0, s>>>((const bf16*)q, q_stride, (const bf16*)k, (const bf16*)v, kv_stride,
                                                      kv_row0, npos, (bf16*)out, hq, hkv, hd, scale, out_tiled);
    else
        attn_rowwise_kernel<float><<<grid, 64, 0, s>>>((const float*)q, q_stride, (const float*)k, (const float*)v,
                                                       kv_stride, kv_row0, npos, (float*)out, hq, hkv, hd, scale, false);
}

}  // namespace vl
