// Row-wise HBM-bound kernels of the decoder block: embedding gather, RMSNorm, rotary embedding, value
// transpose, KV-cache store, hidden-state store.  One workgroup (256 lanes = 4 waves) per token row unless
// noted; loads and stores are contiguous along the row so each wave touches whole cache lines.
#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int ROW_THREADS = 256;

__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < ROW_THREADS / WAVE; ++i) t += red[i];
    __syncthreads();
    return t;
}

// ---------------------------------------------------------------- embedding (S_1 = Embed(x), Section 5.5)
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok,
                                                             const int32_t* __restrict__ row_tok,
                                                             float* __restrict__ resid, uint8_t* __restrict__ valid,
                                                             const int32_t* __restrict__ dst, int d, int vocab) {
    const int64_t n = blockIdx.x;
    int id = tok[row_tok ? row_tok[n] : n];
    if (id < 0 || id >= vocab) {
        id = 0;
        if (valid && threadIdx.x == 0) valid[dst ? dst[n] : n] = 0;
    }
    float* out = resid + n * (int64_t)d;
    const T* src = E + (int64_t)id * d;
    for (int i = threadIdx.x; i < d; i += ROW_THREADS) out[i] = to_f32(src[i]);
}

void launch_embed(const void* E, int dtype, const int32_t* tok, const int32_t* row_tok, float* resid, uint8_t* valid,
                  const int32_t* dst, int64_t rows, int d, int vocab, hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == VL_BF16)
        embed_kernel<bf16><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((const bf16*)E, tok, row_tok, resid, valid, dst, d,
                                                                       vocab);
    else
        embed_kernel<float><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((const float*)E, tok, row_tok, resid, valid, dst,
                                                                        d, vocab);
}

// ---------------------------------------------------------------- RMSNorm
__device__ __forceinline__ void store4(float* o, float a, float b, float c, float d) { *(float4*)o = make_float4(a, b, c, d); }
__device__ __forceinline__ void store4(bf16* o, float a, float b, float c, float d) {
    bf16x4 t;
    t[0] = (bf16)a; t[1] = (bf16)b; t[2] = (bf16)c; t[3] = (bf16)d;
    *(bf16x4*)o = t;
}

template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                               T* __restrict__ out, int d, float eps, bool out_tiled) {
    __shared__ float red[ROW_THREADS / WAVE];
    const int64_t n = blockIdx.x;
    const float4* xr = (const float4*)(x + n * (int64_t)d);
    const float4* g4 = (const float4*)gain;
    const int d4 = d >> 2;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d4; i += ROW_THREADS) {
        const float4 v = xr[i];
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = block_sum(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d4; i += ROW_THREADS) {
        const float4 v = xr[i];
        const float4 g = g4[i];
        T* o = out + (out_tiled ? tiled_off(n, 4 * i, d) : n * (int64_t)d + 4 * i);    // 4 | 32: a quad never straddles a piece
        store4(o, v.x * r * g.x, v.y * r * g.y, v.z * r * g.z, v.w * r * g.w);
    }
}

// One wave per row, the row held in registers between the sum of squares and the scaling (read once): d = 256 * NV.
template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_wave_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                           T* __restrict__ out, int64_t rows, float eps, bool out_tiled) {
    constexpr int D = 256 * NV;
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= rows) return;                                      // whole wave leaves together; no barrier below
    const float4* xr = (const float4*)(x + n * (int64_t)D);
    float4 v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = xr[lane + WAVE * i];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)D + eps);
    const float4* g4 = (const float4*)gain;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = lane + WAVE * i;
        const float4 g = g4[q];
        T* o = out + (out_tiled ? tiled_off(n, 4 * q, D) : n * (int64_t)D + 4 * q);
        store4(o, v[i].x * r * g.x, v[i].y * r * g.y, v[i].z * r * g.z, v[i].w * r * g.w);
    }
}

template <typename T>
static void launch_rmsnorm_t(const float* x, const float* gain, T* out, int64_t rows, int d, float eps, hipStream_t s, bool tiled) {
    const dim3 grid((unsigned)((rows + 3) / 4));
#define VL_RMS(NV) rmsnorm_wave_kernel<T, NV><<<grid, 256, 0, s>>>(x, gain, out, rows, eps, tiled)
    switch ((d & 255) ? 0 : d >> 8) {
        case 1: VL_RMS(1); break;
        case 2: VL_RMS(2); break;
        case 4: VL_RMS(4); break;
        case 8: VL_RMS(8); break;
        case 16: VL_RMS(16); break;
        case 32: VL_RMS(32); break;
        default: rmsnorm_kernel<T><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>(x, gain, out, d, eps, tiled); break;
    }
#undef VL_RMS
}

void launch_rmsnorm(const float* x, const float* gain, void* out, int dtype, int64_t rows, int d, float eps,
                    hipStream_t s, bool out_tiled) {
    if (rows <= 0) return;
    if (dtype == VL_BF16) launch_rmsnorm_t<bf16>(x, gain, (bf16*)out, rows, d, eps, s, out_tiled);
    else launch_rmsnorm_t<float>(x, gain, (float*)out, rows, d, eps, s, false);
}

// ---------------------------------------------------------------- row-major -> tiled image (weights, at load time)
__global__ __launch_bounds__(256) void retile_kernel(const bf16* __restrict__ src, bf16* __restrict__ dst, int64_t rows, int K,
                                                     int64_t row0, int interleave) {
    const int k8 = K >> 3;                                      // 16-byte chunks per row
    const int64_t total = rows * k8;
    for (int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x; id < total; id += (int64_t)gridDim.x * 256) {
        const int64_t r = id / k8;
        const int c = (int)(id - r * k8);
        int64_t dr = row0 + r;
        if (interleave) dr = row0 + 64 * (r >> 5) + (interleave == 2 ? 32 : 0) + (r & 31);
        *(u32x4*)(dst + tiled_off(dr, 8 * c, K)) = *(const u32x4*)(src + r * K + 8 * c);
    }
}

void launch_retile(const void* src, void* dst, int64_t rows, int K, int64_t row0, int interleave, hipStream_t s) {
    if (rows <= 0) return;
    const int64_t total = rows * (K >> 3);
    const unsigned grid = (unsigned)std::min<int64_t>((total + 255) / 256, 65536);
    retile_kernel<<<grid, 256, 0, s>>>((const bf16*)src, (bf16*)dst, rows, K, row0, interleave);
}

// ---------------------------------------------------------------- rotary embedding, in place on Q and K
// With cache_row != NULL the rotated keys and the values of row n are also written to row cache_row[n] of the KV
// cache (kc, vc: [cache rows][hkv*hd]), which saves the token-by-token path a launch per layer.
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void rope_kernel(T* __restrict__ qkv, const int32_t* __restrict__ pos,
                                                            const float2* __restrict__ cs, int hq, int hkv, int hd,
                                                            T* __restrict__ kc, T* __restrict__ vc,
                                                            const int32_t* __restrict__ cache_row) {
    const int64_t n = blockIdx.x;
    const int half = hd >> 1;
    const int p = pos[n];
    T* row = qkv + n * (int64_t)(hq + 2 * hkv) * hd;
    const float2* tab = cs + (int64_t)p * half;
    const int pairs = (hq + hkv) * half;           // query heads then key heads are contiguous in the row
    const int64_t dst = cache_row ? (int64_t)cache_row[n] * hkv * hd : 0;
    for (int i = threadIdx.x; i < pairs; i += ROW_THREADS) {
        const int h = i / half, c = i - h * half;
        const float2 t = tab[c];
        T* a = row + h * hd + c;
        const float x1 = to_f32(a[0]), x2 = to_f32(a[half]);
        const T y1 = from_f32<T>(x1 * t.x - x2 * t.y), y2 = from_f32<T>(x2 * t.x + x1 * t.y);
        a[0] = y1;
        a[half] = y2;
        if (cache_row && h >= hq) {
            T* kd = kc + dst + (h - hq) * hd + c;
            kd[0] = y1;
            kd[half] = y2;
        }
    }
    if (cache_row) {
        const T* vrow = row + (int64_t)(hq + hkv) * hd;
        for (int i = threadIdx.x; i < hkv * hd; i += ROW_THREADS) vc[dst + i] = vrow[i];
    }
}

// bf16 rows whose half head is a multiple of 8: the same rotation on 16-byte vectors (8 pairs per item)
__global__ __launch_bounds__(ROW_THREADS) void rope_vec_kernel(bf16* __restrict__ qkv, const int32_t* __restrict__ pos,
                                                                const float2* __restrict__ cs, int hq, int hkv, int hd,
                                                                bf16* __restrict__ kc, bf16* __restrict__ vc,
                                                                const int32_t* __restrict__ cache_row) {
    const int64_t n = blockIdx.x;
    const int half = hd >> 1, vph = half >> 3;     // vectors per half head
    const int p = pos[n];
    bf16* row = qkv + n * (int64_t)(hq + 2 * hkv) * hd;
    const float2* tab = cs + (int64_t)p * half;
    const int items = (hq + hkv) * vph;
    const int64_t dst = cache_row ? (int64_t)cache_row[n] * hkv * hd : 0;
    for (int i = threadIdx.x; i < items; i += ROW_THREADS) {
        const int h = i / vph, c = (i - h * vph) * 8;
        bf16* a = row + h * hd + c;
        const bf16x8 x1 = *(const bf16x8*)a, x2 = *(const bf16x8*)(a + half);
        bf16x8 y1, y2;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float2 t = tab[c + j];
            const float f1 = (float)x1[j], f2 = (float)x2[j];
            y1[j] = (bf16)(f1 * t.x - f2 * t.y);
            y2[j] = (bf16)(f2 * t.x + f1 * t.y);
        }
        *(bf16x8*)a = y1;
        *(bf16x8*)(a + half) = y2;
        if (cache_row && h >= hq) {
            bf16* kd = kc + dst + (h - hq) * hd + c;
            *(bf16x8*)kd = y1;
            *(bf16x8*)(kd + half) = y2;
        }
    }
    if (cache_row) {
        const bf16* vrow = row + (int64_t)(hq + hkv) * hd;
        for (int i = threadIdx.x * 8; i < hkv * hd; i += ROW_THREADS * 8) *(bf16x8*)(vc + dst + i) = *(const bf16x8*)(vrow + i);
    }
}

void launch_rope(void* qkv, int dtype, const int32_t* pos, const float2* cs, int64_t rows, int hq, int hkv, int hd,
                 hipStream_t s, void* kcache, void* vcache, const int32_t* cache_row) {
    if (rows <= 0) return;
    if (dtype == VL_BF16 && (hd & 15) == 0)
        rope_vec_kernel<<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((bf16*)qkv, pos, cs, hq, hkv, hd, (bf16*)kcache, (bf16*)vcache,
                                                                     cache_row);
    else if (dtype == VL_BF16)
        rope_kernel<bf16><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((bf16*)qkv, pos, cs, hq, hkv, hd, (bf16*)kcache,
                                                                      (bf16*)vcache, cache_row);
    else
        rope_kernel<float><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((float*)qkv, pos, cs, hq, hkv, hd, (float*)kcache,
                                                                       (float*)vcache, cache_row);
}

// ---------------------------------------------------------------- V transpose for the matrix-core attention
// Tile of 64 tokens x 64 channels through LDS so that both the read (along channels) and the write
// (along tokens) are contiguous.  grid = (ceil(rows/64), hkv*hd/64).
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ vt,
                                                           const int32_t* __restrict__ vt_col, int64_t rows, int hq,
                                                           int hkv, int hd, int64_t ldv) {
    __shared__ bf16 tile[64][66];
    __shared__ int32_t cols[64];
    const int64_t n0 = (int64_t)blockIdx.x * 64;
    const int c0 = blockIdx.y * 64;                      // channel offset within the hkv*hd value block
    const int64_t pitch = (int64_t)(hq + 2 * hkv) * hd;
    const bf16* vbase = qkv + (int64_t)(hq + hkv) * hd + c0;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    if (threadIdx.x < 64) cols[threadIdx.x] = (n0 + threadIdx.x < rows) ? vt_col[n0 + threadIdx.x] : -1;
    for (int r = ty; r < 64; r += 4) {
        const int64_t n = n0 + r;
        tile[r][tx] = (n < rows) ? vbase[n * pitch + tx] : (bf16)0.f;
    }
    __syncthreads();
    // consecutive tokens of one sequence have consecutive vt columns, so lanes write contiguous runs
    for (int c = ty; c < 64; c += 4) {
        const int col = cols[tx];
        if (col >= 0) vt[(int64_t)(c0 + c) * ldv + col] = tile[tx][c];
    }
}

void launch_transpose_v(const void* qkv, void* vt, const int32_t* vt_col, int64_t rows, int hq, int hkv, int hd,
                        int64_t ldv, hipStream_t s) {
    if (rows <= 0) return;
    dim3 grid((unsigned)((rows + 63) / 64), (unsigned)(hkv * hd / 64));
    transpose_v_kernel<<<grid, 256, 0, s>>>((const bf16*)qkv, (bf16*)vt, vt_col, rows, hq, hkv, hd, ldv);
}

// ---------------------------------------------------------------- hidden-state store (commitments out)
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void store_hidden_kernel(const float* __restrict__ resid, T* __restrict__ out,
                                                                    const int32_t* __restrict__ dst, int d) {
    const int64_t n = blockIdx.x;
    const int64_t o = dst ? (int64_t)dst[n] : n;
    const float* src = resid + n * (int64_t)d;
    T* dp = out + o * (int64_t)d;
    for (int i = threadIdx.x; i < d; i += ROW_THREADS) dp[i] = from_f32<T>(src[i]);
}

void launch_store_hidden(const float* resid, void* out, int dtype, const int32_t* dst, int64_t rows, int d,
                         hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == VL_BF16)
        store_hidden_kernel<bf16><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>(resid, (bf16*)out, dst, d);
    else
        store_hidden_kernel<float><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>(resid, (float*)out, dst, d);
}

// ---------------------------------------------------------------- recorded states in (a segment's starting point)
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void load_hidden_kernel(const T* __restrict__ in, float* __restrict__ resid, int d) {
    const int64_t n = blockIdx.x;
    const T* src = in + n * (int64_t)d;
    float* dp = resid + n * (int64_t)d;
    for (int i = threadIdx.x; i < d; i += ROW_THREADS) dp[i] = to_f32(src[i]);
}

void launch_load_hidden(const void* in, int dtype, float* resid, int64_t rows, int d, hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == VL_BF16)
        load_hidden_kernel<bf16><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((const bf16*)in, resid, d);
    else
        load_hidden_kernel<float><<<dim3((unsigned)rows), ROW_THREADS, 0, s>>>((const float*)in, resid, d);
}

// ---------------------------------------------------------------- per-step index slices of the token-by-token path
// cur[k * stride + i] = array_k[off + i] for the four index arrays, then off += rows.  One workgroup; every lane reads
// the offset before lane 0 advances it.
__global__ __launch_bounds__(256) void step_prologue_kernel(const int32_t* __restrict__ a0, const int32_t* __restrict__ a1,
                                                            const int32_t* __restrict__ a2, const int32_t* __restrict__ a3,
                                                            int32_t* __restrict__ cur, int32_t* __restrict__ off, int rows,
                                                            int stride) {
    const int o = *off;
    __syncthreads();
    for (int i = threadIdx.x; i < rows; i += 256) {
        cur[i] = a0[o + i];
        cur[stride + i] = a1[o + i];
        cur[2 * stride + i] = a2[o + i];
        cur[3 * stride + i] = a3[o + i];
    }
    if (threadIdx.x == 0) *off = o + rows;
}

void launch_step_prologue(const int32_t* a0, const int32_t* a1, const int32_t* a2, const int32_t* a3, int32_t* cur, int32_t* off,
                          int rows, int stride, hipStream_t s) {
    step_prologue_kernel<<<1, 256, 0, s>>>(a0, a1, a2, a3, cur, off, rows, stride);
}

__global__ void scatter_i32_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ out,
                                   const int32_t* __restrict__ dst, int64_t rows) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) out[dst ? dst[i] : i] = src[i];
}

void launch_scatter_i32(const int32_t* src, int32_t* out, const int32_t* dst, int64_t rows, hipStream_t s) {
    if (rows <= 0) return;
    scatter_i32_kernel<<<dim3((unsigned)((rows + 255) / 256)), 256, 0, s>>>(src, out, dst, rows);
}

__global__ void fill_u8_kernel(uint8_t* p, uint8_t v, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

void launch_fill_u8(uint8_t* p, uint8_t v, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    fill_u8_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>(p, v, n);
}

}  // namespace vl
