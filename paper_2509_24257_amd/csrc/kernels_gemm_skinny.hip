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
//               For the q/k/v projection of a decode step the two row groups are 16 channels of a head and their
//               rotary partners half a head further on: the epilogue rounds to bf16, rotates query and key pairs by
//               the row's position and appends keys and values to the KV cache, which saves the step a launch per layer.
//   RMSNorm   : with XS > 0 the operand A is the fp32 residual stream: every workgroup first normalises the (<= 16) rows
//               into LDS as bf16, one wave per row with the sums taken in the order of the stand-alone kernel, while its
//               first weight loads are in flight, and then reads the A fragments from there.  The rows come out of L2;
//               this replaces a launch whose whole cost was its latency.  Used for the q/k/v projection, whose grid is
//               one workgroup per compute unit; for the gate/up projection (3.5 workgroups per compute unit, each
//               repeating the rows' two round trips) it measured 4 us slower than the separate kernel.
#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int GS_THREADS = 512;
constexpr int GS_WAVES = 8;
#ifndef GS_UNROLL
#define GS_UNROLL 4
#endif

// what the rotary epilogue needs: positions and cache rows per row of A, the cos/sin table [position][hd/2], the caches
struct RopeArgs {
    const int32_t* pos;
    const int32_t* cache_row;
    const float2* cs;
    bf16 *kc, *vc;
    int hq, hkv, hd;
};

struct NormArgs {
    const float* gain;
    float eps;
};
// bytes of LDS for the normalised rows: row pitch 2 K + 16 (the 16 spread the rows of a fragment read over the banks)
constexpr int GS_XS = 8 * (2 * 4096 + 16);                   // 8 rows of 4096 channels
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

template <int EPI, int MT, int NG, int XS = 0>
__global__ __launch_bounds__(GS_THREADS) void gemm_skinny_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                                                                 int M, int N, int K, void* __restrict__ outp, int layout,
                                                                 RopeArgs ra, NormArgs na) {
    static_assert(XS == 0 || MT == 1, "the fused RMSNorm holds at most 16 rows");
    __shared__ __align__(16) unsigned char xs[XS > 0 ? XS : 16];
    static_assert(EPI != EPI_SWIGLU || NG == 2, "SwiGLU pairs a gate group with an up group");
    static_assert(EPI != EPI_QKV_ROPE || NG == 2, "the rotary epilogue pairs a group of channels with its partners");
    // partial tiles of the eight waves; with XS > 0 they reuse the rows' LDS once the main loop is done with it
    __shared__ __align__(16) float red_own[XS > 0 ? 1 : GS_WAVES][NG * MT * 256];
    static_assert(XS == 0 || XS >= (int)sizeof(float) * GS_WAVES * NG * MT * 256, "the rows' buffer also holds the partial tiles");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    int r0, r1, ch0 = 0;                                        // first W row of each group; first output channel (SwiGLU)
    if (EPI == EPI_SWIGLU) {
        const int b = blockIdx.x >> 1, h = blockIdx.x & 1;
        r0 = b * 64 + h * 16;
        r1 = r0 + 32;
        ch0 = b * 32 + h * 16;
    } else if (EPI == EPI_QKV_ROPE) {
        const int half = ra.hd >> 1, bph = half >> 4;           // 16-channel blocks per half head
        const int head = blockIdx.x / bph;
        ch0 = (blockIdx.x - head * bph) * 16;                   // first channel within the head
        r0 = head * ra.hd + ch0;
        r1 = r0 + half;
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
    const int x_pitch = 2 * K + 16, x_off = min(fr, M - 1) * x_pitch + fq * 16;     // XS > 0: byte offsets into xs
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
    // two register stages of U k-steps each: the loads of one stage are in flight while the other feeds the MFMAs, so a
    // wave never sits out a whole memory round trip between two bursts of loads
    constexpr int U = GS_UNROLL;
    bf16x8 a0[2][U], a1[2][U], b[2][MT][U];
    auto load_w = [&](int st, int k0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t ow = (k0 + u) * w_step;
            a0[st][u] = *(const bf16x8*)(w0 + ow);
            if (NG == 2) a1[st][u] = *(const bf16x8*)(w1 + ow);
        }
    };
    // A fragments: from memory they travel with the weights of their stage; from LDS (XS > 0) they are read when the
    // stage is used, which keeps the kernel at two workgroups per compute unit
    auto load_b = [&](int st, int k0) {
        if (XS > 0) return;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) b[st][t][u] = *(const bf16x8*)(ap[t] + (k0 + u) * a_step);
    };
    auto load_stage = [&](int st, int k0) {
        load_w(st, k0);
        load_b(st, k0);
    };
    auto mma_stage = [&](int st, int k0) {
        if (XS > 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) b[st][0][u] = *(const bf16x8*)(xs + x_off + (k0 + u) * 64);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[st][u], b[st][t][u], acc[0][t], 0, 0, 0);
                if (NG == 2) acc[NG - 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[st][u], b[st][t][u], acc[NG - 1][t], 0, 0, 0);
            }
    };
    const int n_it = (ke - ks) / U;
    if (n_it > 0) load_w(0, ks);
    if (XS > 0) {
        __builtin_amdgcn_sched_barrier(0);                      // the weight loads above go out first
        const int k4 = K >> 2;
        const float4* g4 = (const float4*)na.gain;
        // the row is wave-uniform and said to be: addresses are then a scalar base plus one per-lane offset
        for (int row = __builtin_amdgcn_readfirstlane(wave); row < M; row += GS_WAVES) {
            const float4* xr = (const float4*)((const float*)A + (int64_t)row * K);
            // K / 4 is a multiple of 64, so a whole wave is inside or outside the row together; the loads of a batch go out
            // back to back (a chunk past the end re-reads the last one and is not used)
            float ss = 0.f;
            constexpr int PB = 16;                              // loads per batch: a row of 4096 is one batch
            for (int c0 = 0; c0 < k4; c0 += WAVE * PB) {       // c0 and every condition on it are wave-uniform
                float4 v[PB];
#pragma unroll
                for (int j = 0; j < PB; ++j) v[j] = (xr + min(c0 + WAVE * j, k4 - WAVE))[lane];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < PB; ++j)
                    if (c0 + WAVE * j < k4) ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
            }
            ss = wave_sum(ss);
            const float r = 1.0f / sqrtf(ss / (float)K + na.eps);
            for (int c0 = 0; c0 < k4; c0 += WAVE * PB) {
                float4 v[PB], g[PB];
#pragma unroll
                for (int j = 0; j < PB; ++j) {
                    const int i = min(c0 + WAVE * j, k4 - WAVE);
                    v[j] = (xr + i)[lane];
                    g[j] = (g4 + i)[lane];
                }
#pragma unroll
                for (int j = 0; j < PB; ++j)                     // all loads of the batch are issued here, none inside a branch below
                    asm volatile("" : "+v"(v[j].x), "+v"(v[j].y), "+v"(v[j].z), "+v"(v[j].w), "+v"(g[j].x), "+v"(g[j].y), "+v"(g[j].z),
                                 "+v"(g[j].w));
#pragma unroll
                for (int j = 0; j < PB; ++j)
                    if (c0 + WAVE * j < k4)
                        *(bf16x4*)(xs + row * x_pitch + (c0 + WAVE * j + lane) * 8) =
                            bf16x4{(bf16)(v[j].x * r * g[j].x), (bf16)(v[j].y * r * g[j].y), (bf16)(v[j].z * r * g[j].z),
                                   (bf16)(v[j].w * r * g[j].w)};
            }
        }
        __syncthreads();
    }
    if (n_it > 0) load_b(0, ks);
    int it = 0;
    for (; it + 2 < n_it; it += 2) {                            // branch-free body: the wait counts stay exact
        load_stage(1, ks + (it + 1) * U);
        __builtin_amdgcn_sched_barrier(0);                      // keep the loads ahead of the MFMAs they overlap
        mma_stage(0, ks + it * U);
        __builtin_amdgcn_sched_barrier(0);
        load_stage(0, ks + (it + 2) * U);
        __builtin_amdgcn_sched_barrier(0);
        mma_stage(1, ks + (it + 1) * U);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (n_it - it == 2) {                                       // wave-uniform
        load_stage(1, ks + (it + 1) * U);
        mma_stage(0, ks + it * U);
        mma_stage(1, ks + (it + 1) * U);
    } else if (n_it - it == 1) {
        mma_stage(0, ks + it * U);
    }
    ks += n_it * U;
    for (; ks < ke; ++ks) {
        const int64_t ow = ks * w_step, oa = ks * a_step;
        const bf16x8 wa = *(const bf16x8*)(w0 + ow), wb = *(const bf16x8*)((NG == 2 ? w1 : w0) + ow);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const bf16x8 bb = XS > 0 ? *(const bf16x8*)(xs + x_off + ks * 64) : *(const bf16x8*)(ap[t] + oa);
            acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, bb, acc[0][t], 0, 0, 0);
            if (NG == 2) acc[NG - 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, bb, acc[NG - 1][t], 0, 0, 0);
        }
    }
    float (*red)[NG * MT * 256] = XS > 0 ? (float (*)[NG * MT * 256]) xs : red_own;
    if (XS > 0) __syncthreads();                                // every wave has read its last fragment from xs
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
                ((bf16*)outp)[(layout & GL_OUT_TILED) ? tiled_off(m, f, F) : (int64_t)m * F + f] = (bf16)silu_mul(g, u);
        }
    } else if (EPI == EPI_QKV_ROPE) {
        const int half = ra.hd >> 1, head = r0 / ra.hd;
        const int64_t kvd = (int64_t)ra.hkv * ra.hd;
        for (int e = threadIdx.x; e < PER_GROUP; e += GS_THREADS) {
            float x1 = 0.f, x2 = 0.f;
#pragma unroll
            for (int w = 0; w < GS_WAVES; ++w) {
                x1 += red[w][e];
                x2 += red[w][PER_GROUP + e];
            }
            const int l = (e & 255) >> 2, r = e & 3;
            const int m = (e >> 8) * 16 + (l & 15), c = ch0 + 4 * (l >> 4) + r;
            if (m >= M) continue;
            bf16 y1 = (bf16)x1, y2 = (bf16)x2;                  // the projection's own rounding comes first
            if (head < ra.hq + ra.hkv) {
                const float2 t = ra.cs[(int64_t)ra.pos[m] * half + c];
                const float f1 = (float)y1, f2 = (float)y2;
                y1 = (bf16)(f1 * t.x - f2 * t.y);
                y2 = (bf16)(f2 * t.x + f1 * t.y);
            }
            bf16* o = (bf16*)outp + (int64_t)m * N + r0 + 4 * (l >> 4) + r;
            o[0] = y1;
            o[half] = y2;
            if (head >= ra.hq) {
                const bool is_k = head < ra.hq + ra.hkv;
                bf16* d = (is_k ? ra.kc : ra.vc) + (int64_t)ra.cache_row[m] * kvd + (head - ra.hq - (is_k ? 0 : ra.hkv)) * ra.hd + c;
                d[0] = y1;
                d[half] = y2;
            }
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
    const RopeArgs none{};
    const NormArgs plain{};
    if (M <= 16) gemm_skinny_kernel<EPI, 1, NG><<<grid, GS_THREADS, 0, s>>>(A, W, M, N, K, out, layout, none, plain);
    else if (M <= 32) gemm_skinny_kernel<EPI, 2, NG><<<grid, GS_THREADS, 0, s>>>(A, W, M, N, K, out, layout, none, plain);
    else gemm_skinny_kernel<EPI, 4, NG><<<grid, GS_THREADS, 0, s>>>(A, W, M, N, K, out, layout, none, plain);
}

bool gemm_skinny_norm_supported(int M, int K) { return M >= 1 && M <= 16 && (K & 255) == 0 && (int64_t)M * (2 * K + 16) <= GS_XS; }

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

bool gemm_skinny_qkv_rope_supported(int M, int hd) { return M <= GEMM_SKINNY_MAX_M && (hd & 31) == 0; }

void launch_gemm_skinny_qkv_rope(const void* A, const void* W, int M, int K, void* qkv, const int32_t* pos, const float2* cs,
                                 const int32_t* cache_row, void* kcache, void* vcache, int hq, int hkv, int hd, hipStream_t s,
                                 int layout, const float* norm_gain, float eps) {
    if (M <= 0) return;
    const int N = (hq + 2 * hkv) * hd;
    const RopeArgs ra{pos, cache_row, cs, (bf16*)kcache, (bf16*)vcache, hq, hkv, hd};
    if (norm_gain) {
        // A = fp32 rows that the kernel normalises itself (see the header)
        gemm_skinny_kernel<EPI_QKV_ROPE, 1, 2, GS_XS><<<(unsigned)(N / 32), GS_THREADS, 0, s>>>((const bf16*)A, (const bf16*)W, M, N, K, qkv,
                                                                                              layout, ra, NormArgs{norm_gain, eps});
        return;
    }
    const NormArgs plain{};
    const unsigned grid = (unsigned)(N / 32);                   // a workgroup owns 16 channels and their 16 partners
    const bf16 *a = (const bf16*)A, *w = (const bf16*)W;
    if (M <= 16) gemm_skinny_kernel<EPI_QKV_ROPE, 1, 2><<<grid, GS_THREADS, 0, s>>>(a, w, M, N, K, qkv, layout, ra, plain);
    else if (M <= 32) gemm_skinny_kernel<EPI_QKV_ROPE, 2, 2><<<grid, GS_THREADS, 0, s>>>(a, w, M, N, K, qkv, layout, ra, plain);
    else gemm_skinny_kernel<EPI_QKV_ROPE, 4, 2><<<grid, GS_THREADS, 0, s>>>(a, w, M, N, K, qkv, layout, ra, plain);
}

}  // namespace vl
