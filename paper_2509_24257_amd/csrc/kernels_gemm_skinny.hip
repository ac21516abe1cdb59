// C[M,N] = A[M,K] * W[N,K]^T for M <= 64 rows: the GEMM of the token-by-token path (Section 5.5), where a step
// carries one row per live sequence and the whole cost is streaming W out of HBM once.
//
//   workgroup : 512 lanes = 8 waves; owns NG groups of 16 rows of W (two for wide matrices and for SwiGLU, one when N
//               is small, so that the grid still covers the chip) and all M rows of A
//   split K   : wave w reduces its own eighth of K, so that even N = 4096 puts 1024 waves and ~12 x 16 B per lane of
//               loads in flight; the eight partial tiles meet in LDS and are summed in wave order (fixed, so the
//               result is bit-reproducible)
//   MFMA      : v_mfma_f32_16x16x32_bf16 with W as the 16-row operand and A (transposed) as the 16-column operand:
//               lane l feeds W[row l%16][k 8*(l/16) .. +7] and A[row l%16][same k], and receives
//               C^T[w-row 4*(l/16) + r][a-row l%16], r = 0..3.  Rows of A beyond M repeat row M-1 and are never stored.
//   loads     : every lane reads 16 contiguous bytes; the four k-steps of one unrolled iteration cover 256 contiguous
//               bytes of every W row
//   epilogues : as in the large-tile kernel; for SwiGLU the two row groups are the gate rows and the up rows of the
//               same 16 channels (W interleaves 32 gate rows, 32 up rows), so silu(gate) * up is formed in place.
#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int GS_THREADS = 512;
constexpr int GS_WAVES = 8;

template <int EPI, int MT, int NG>
__global__ __launch_bounds__(GS_THREADS) void gemm_skinny_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                                                                 int M, int N, int K, void* __restrict__ outp, int layout) {
    static_assert(EPI != EPI_SWIGLU || NG == 2, "SwiGLU pairs a gate group with an up group");
    __shared__ __align__(16) float red[GS_WAVES][NG * MT * 256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    int r0, r1, ch0 = 0;                                        // first W row of each group; first output channel (SwiGLU)
    if (EPI == EPI_SWIGLU) {
        const int b = blockIdx.x >> 1, h = blockIdx.x & 1;
        r0 = b * 64 + h * 16;
        r1 = r0 + 32;
        ch0 = b * 32 + h * 16;
    } else {
        r0 = blockIdx.x * (16 * NG);
        r1 = r0 + 16;
    }
    // operands are row-major or tiled images (see tiled_off); a k-step of 32 is then 32 or 8192 elements further on
    const bool wt = layout & GL_W_TILED, at = layout & GL_A_TILED;
    const int64_t w_step = wt ? TL_PIECE : 32, a_step = at ? TL_PIECE : 32;
    const int wr0 = min(r0 + fr, N - 1), wr1 = min(r1 + fr, N - 1);
    const bf16* w0 = W + (wt ? tiled_off(wr0, 0, K) : (int64_t)wr0 * K) + fq * 8;
    const bf16* w1 = W + (wt ? tiled_off(wr1, 0, K) : (int64_t)wr1 * K) + fq * 8;
    const bf16* ap[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int ar = min(t * 16 + fr, M - 1);
        ap[t] = A + (at ? tiled_off(ar, 0, K) : (int64_t)ar * K) + fq * 8;
    }

    f32x4 acc[NG][MT];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[g][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int steps = K >> 5;                                   // k-steps of 32
    int ks = (int)(((int64_t)steps * wave) / GS_WAVES);
    const int ke = (int)(((int64_t)steps * (wave + 1)) / GS_WAVES);
    for (; ks + 4 <= ke; ks += 4) {
        bf16x8 a0[4], a1[4], b[MT][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t ow = (ks + u) * w_step, oa = (ks + u) * a_step;
            a0[u] = *(const bf16x8*)(w0 + ow);
            if (NG == 2) a1[u] = *(const bf16x8*)(w1 + ow);
#pragma unroll
            for (int t = 0; t < MT; ++t) b[t][u] = *(const bf16x8*)(ap[t] + oa);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[u], b[t][u], acc[0][t], 0, 0, 0);
                if (NG == 2) acc[NG - 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[u], b[t][u], acc[NG - 1][t], 0, 0, 0);
            }
    }
    for (; ks < ke; ++ks) {
        const int64_t ow = ks * w_step, oa = ks * a_step;
        const bf16x8 a0 = *(const bf16x8*)(w0 + ow), a1 = *(const bf16x8*)((NG == 2 ? w1 : w0) + ow);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const bf16x8 b = *(const bf16x8*)(ap[t] + oa);
            acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc[0][t], 0, 0, 0);
            if (NG == 2) acc[NG - 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc[NG - 1][t], 0, 0, 0);
        }
    }
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < MT; ++t) *(f32x4*)&red[wave][((g * MT + t) * 64 + lane) * 4] = acc[g][t];
    __syncthreads();

    // element e of a group: a-row tile t = e / 256, lane l = (e % 256) / 4, r = e % 4 -> w-row 4*(l/16) + r, a-row 16 t + l%16
    constexpr int PER_GROUP = MT * 256;
    if (EPI == EPI_SWIGLU) {
        const int F = N >> 1;
        for (int e = threadIdx.x; e < PER_GROUP; e += GS_THREADS) {
            float g = 0.f, u = 0.f;
#pragma unroll
            for (int w = 0; w < GS_WAVES; ++w) {
                g += red[w][e];
                u += red[w][PER_GROUP + e];
            }
            const int l = (e & 255) >> 2, r = e & 3;
            const int m = (e >> 8) * 16 + (l & 15), f = ch0 + 4 * (l >> 4) + r;
            if (m < M && f < F)
                ((bf16*)outp)[(layout & GL_OUT_TILED) ? tiled_off(m, f, F) : (int64_t)m * F + f] = (bf16)(g / (1.0f + __expf(-g)) * u);
        }
    } else {
        for (int e = threadIdx.x; e < NG * PER_GROUP; e += GS_THREADS) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < GS_WAVES; ++w) v += red[w][e];
            const int grp = e / PER_GROUP, ee = e - grp * PER_GROUP;
            const int l = (ee & 255) >> 2, r = ee & 3;
            const int m = (ee >> 8) * 16 + (l & 15), n = (grp ? r1 : r0) + 4 * (l >> 4) + r;
            if (m < M && n < N) {
                const int64_t o = (int64_t)m * N + n;
                if (EPI == EPI_STORE) ((bf16*)outp)[o] = (bf16)v;
                if (EPI == EPI_STORE_F32) ((float*)outp)[o] = v;
                if (EPI == EPI_ADD_RESID) ((float*)outp)[o] += v;
            }
        }
    }
}

template <int EPI, int NG>
static void launch_mt(const bf16* A, const bf16* W, int M, int N, int K, void* out, hipStream_t s, int layout) {
    const unsigned grid = (unsigned)((N + 16 * NG - 1) / (16 * NG));
    if (M <= 16) gemm_skinny_kernel<EPI, 1, NG><<<grid, GS_THREADS, 0, s>>>(A, W, M, N, K, out, layout);
    else if (M <= 32) gemm_skinny_kernel<EPI, 2, NG><<<grid, GS_THREADS, 0, s>>>(A, W, M, N, K, out, layout);
    else gemm_skinny_kernel<EPI, 4, NG><<<grid, GS_THREADS, 0, s>>>(A, W, M, N, K, out, layout);
}

// one row group per workgroup while two would leave fewer than two workgroups per compute unit
template <int EPI>
static void launch_ng(const bf16* A, const bf16* W, int M, int N, int K, void* out, hipStream_t s, int layout) {
    if (EPI == EPI_SWIGLU || N >= 32 * 512) launch_mt<EPI, 2>(A, W, M, N, K, out, s, layout);
    else launch_mt<EPI == EPI_SWIGLU ? EPI_STORE : EPI, 1>(A, W, M, N, K, out, s, layout);
}

void launch_gemm_skinny(const void* A, const void* W, int M, int N, int K, int epi, void* out, hipStream_t s, int layout) {
    if (M <= 0 || N <= 0) return;
    const bf16* a = (const bf16*)A;
    const bf16* w = (const bf16*)W;
    switch (epi) {
        case EPI_STORE: launch_ng<EPI_STORE>(a, w, M, N, K, out, s, layout); break;
        case EPI_STORE_F32: launch_ng<EPI_STORE_F32>(a, w, M, N, K, out, s, layout); break;
        case EPI_ADD_RESID: launch_ng<EPI_ADD_RESID>(a, w, M, N, K, out, s, layout); break;
        default: launch_ng<EPI_SWIGLU>(a, w, M, N, K, out, s, layout); break;
    }
}

}  // namespace vl
