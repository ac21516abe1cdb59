// C[M,N] = A[M,K] * W[N,K]^T on the vector ALUs: 64x64 output tile per 256-lane workgroup, K stepped by 16
// through LDS, each lane owns a 4x4 block of outputs, fp32 accumulation.  This is the GEMM of the fp32
// model path and of the token-by-token decode path (M = a handful of rows); the bf16 prefill GEMMs run on
// the matrix cores instead (kernels_gemm_mfma.hip).
#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int SG_BM = 64, SG_BN = 64, SG_BK = 16;

template <typename T> struct Vec4Load;
template <> struct Vec4Load<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
        const float4 t = *(const float4*)p;
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
};
template <> struct Vec4Load<bf16> {
    static __device__ __forceinline__ void load(const bf16* p, float (&v)[4]) {
        const bf16x4 t = *(const bf16x4*)p;
        v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
    }
};

template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const T* __restrict__ A, const T* __restrict__ W, int M, int N,
                                                          int K, void* __restrict__ outp, int ib) {
    __shared__ float As[SG_BK][SG_BM + 4];
    __shared__ float Ws[SG_BK][SG_BN + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * SG_BM, n0 = blockIdx.x * SG_BN;
    const int lr = tid >> 2, lk = (tid & 3) * 4;          // this lane loads row lr, k offset lk..lk+3 of each tile
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += SG_BK) {
        float a[4] = {0.f, 0.f, 0.f, 0.f}, w[4] = {0.f, 0.f, 0.f, 0.f};
        if (m0 + lr < M && k0 + lk < K) Vec4Load<T>::load(A + (int64_t)(m0 + lr) * K + k0 + lk, a);
        if (n0 + lr < N && k0 + lk < K) Vec4Load<T>::load(W + (int64_t)(n0 + lr) * K + k0 + lk, w);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            As[lk + i][lr] = a[i];
            Ws[lk + i][lr] = w[i];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < SG_BK; ++kk) {
            float av[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = Ws[kk][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty + 16 * i;
        if (m >= M) continue;
        if (EPI == EPI_SWIGLU) {
            T* out = (T*)outp;
            const int F = N >> 1;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                // ib == 16: (gate, up) = columns (j, j+1) for j in {0, 2};  ib == 32: (j, j+2) for j in {0, 1}
                const int jg = (ib == 16) ? 2 * p : p;
                const int ju = (ib == 16) ? 2 * p + 1 : p + 2;
                const int f = (n0 >> 1) + 16 * p + tx;
                if (f < F) {
                    const float g = acc[i][jg], u = acc[i][ju];
                    out[(int64_t)m * F + f] = from_f32<T>(g / (1.0f + expf(-g)) * u);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx + 16 * j;
                if (n >= N) continue;
                const int64_t o = (int64_t)m * N + n;
                if (EPI == EPI_STORE) ((T*)outp)[o] = from_f32<T>(acc[i][j]);
                if (EPI == EPI_STORE_F32) ((float*)outp)[o] = acc[i][j];
                if (EPI == EPI_ADD_RESID) ((float*)outp)[o] += acc[i][j];
            }
        }
    }
}

template <typename T>
static void dispatch(const void* A, const void* W, int M, int N, int K, int epi, void* out, int ib, hipStream_t s) {
    dim3 grid((unsigned)((N + SG_BN - 1) / SG_BN), (unsigned)((M + SG_BM - 1) / SG_BM));
    const T* a = (const T*)A;
    const T* w = (const T*)W;
    switch (epi) {
        case EPI_STORE: gemm_simple_kernel<T, EPI_STORE><<<grid, 256, 0, s>>>(a, w, M, N, K, out, ib); break;
        case EPI_STORE_F32: gemm_simple_kernel<T, EPI_STORE_F32><<<grid, 256, 0, s>>>(a, w, M, N, K, out, ib); break;
        case EPI_ADD_RESID: gemm_simple_kernel<T, EPI_ADD_RESID><<<grid, 256, 0, s>>>(a, w, M, N, K, out, ib); break;
        default: gemm_simple_kernel<T, EPI_SWIGLU><<<grid, 256, 0, s>>>(a, w, M, N, K, out, ib); break;
    }
}

void launch_gemm_simple(const void* A, const void* W, int dtype, int M, int N, int K, int epi, void* out, int ib,
                        hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    if (dtype == VL_BF16) dispatch<bf16>(A, W, M, N, K, epi, out, ib, s);
    else dispatch<float>(A, W, M, N, K, epi, out, ib, s);
}

}  // namespace vl
