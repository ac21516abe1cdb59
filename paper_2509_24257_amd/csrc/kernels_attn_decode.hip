// Attention of the token-by-token path (Section 5.5): one query position per live sequence against that sequence's
// KV cache.  One workgroup (8 waves) per (query row, G query heads that share one KV head).  With many rows G is the
// whole group Hq / Hkv, so every cached key and value is read once; with few rows (a step of 8 sequences gives only 64
// such workgroups, and the score and value arithmetic of four heads in one wave is what the step then waits for) the
// group is split over several workgroups, which re-read the keys and values through the L2 they share.
//
//   keys    : walked 64 at a time, block kb by wave kb % 8.  A key row (head_dim bf16) is read by head_dim/8 adjacent
//             lanes, 16 bytes each, so a load instruction covers whole rows; each lane multiplies its 8 channels with
//             the matching 8 query channels it keeps in registers, and a butterfly over the lanes of a row completes
//             the dot product.  After head_dim/8 such passes lane l holds the score of key
//             (l % LPK) * KPP + l / LPK of the block (LPK lanes per key, KPP keys per pass).
//   softmax : online, per wave, in fp32 (running maximum and sum per query head).
//   values  : per key one coalesced row read (lane l owns channels l*DPL .. +DPL-1); the key's probability is
//             broadcast from the lane that holds it.  Row reads are issued in batches ahead of their use.
//   combine : the eight waves' (max, sum, weighted values) meet in LDS and are merged in wave order.
#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int AD_THREADS = 512;
constexpr int AD_WAVES = 8;
constexpr int AD_FILL = 256;                                   // workgroups wanted: one per compute unit

// DPL consecutive bf16 channels of one value row, held as loaded
template <int DPL> struct VLoad;
template <> struct VLoad<1> {
    bf16 x;
    __device__ __forceinline__ void load(const bf16* p) { x = *p; }
    __device__ __forceinline__ float get(int) const { return (float)x; }
};
template <> struct VLoad<2> {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 x;
    __device__ __forceinline__ void load(const bf16* p) { x = *(const bf16x2*)p; }
    __device__ __forceinline__ float get(int i) const { return (float)x[i]; }
};

template <int G, int HD>
__global__ __launch_bounds__(AD_THREADS) void attn_decode_kernel(const bf16* __restrict__ q, int64_t q_stride,
                                                                 const bf16* __restrict__ k, const bf16* __restrict__ v,
                                                                 int64_t kv_stride, const int32_t* __restrict__ kv_row0,
                                                                 const int32_t* __restrict__ npos, bf16* __restrict__ out,
                                                                 int hq, int kv_group, float scale, bool out_tiled) {
    constexpr int LPK = HD / 8;                                 // lanes per key row
    constexpr int KPP = WAVE / LPK;                             // keys per pass
    constexpr int DPL = HD / WAVE;                              // value channels per lane
    constexpr int KCH = (G >= 8 && LPK > 8) ? 8 : LPK;          // key passes requested together
    constexpr int VCH = G >= 8 ? 16 : (G >= 4 ? 32 : 64);       // value rows requested together
    __shared__ float part_o[AD_WAVES][G][HD];
    __shared__ float part_m[AD_WAVES][G], part_l[AD_WAVES][G];
    const int64_t row = blockIdx.x;
    const int qh0 = blockIdx.y * G, kvh = qh0 / kv_group;      // first query head of this workgroup, its KV head
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nkeys = npos[row] + 1;
    const int64_t base = (int64_t)kv_row0[row];
    const int sub = lane % LPK, kin = lane / LPK;               // 16-byte piece of a row, key within a pass

    float qr[G][8];                                             // this lane's 8 channels of every query head, pre-scaled
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const bf16x8 t = *(const bf16x8*)(q + row * q_stride + (int64_t)(qh0 + g) * HD + sub * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) qr[g][i] = (float)t[i] * scale;
    }
    float m[G], l[G], o[G][DPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < DPL; ++i) o[g][i] = 0.f;
    }

    const int nblocks = (nkeys + WAVE - 1) / WAVE;
    for (int kb = wave; kb < nblocks; kb += AD_WAVES) {
        const int t0 = kb * WAVE;
        // ---- loads go out in batches well ahead of their use (the step is latency-bound: few workgroups, short
        // loops); the batch sizes keep the kernel inside the register file.  Rows past the last key re-read it and are
        // masked below.  The first batch of value rows is requested before the scores are computed.
        const bf16* vp = v + base * kv_stride + (int64_t)kvh * HD + lane * DPL;
        VLoad<DPL> vr[VCH];
#pragma unroll
        for (int jj = 0; jj < VCH; ++jj) vr[jj].load(vp + (int64_t)min(t0 + jj, nkeys - 1) * kv_stride);
        // ---- scores: pass j covers keys t0 + j*KPP .. + KPP-1
        float sc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) sc[g] = -INFINITY;
#pragma unroll
        for (int jc = 0; jc < LPK; jc += KCH) {
            bf16x8 kreg[KCH];
#pragma unroll
            for (int j = 0; j < KCH; ++j) {
                const int t = t0 + (jc + j) * KPP + kin;
                kreg[j] = *(const bf16x8*)(k + (base + min(t, nkeys - 1)) * kv_stride + (int64_t)kvh * HD + sub * 8);
            }
#pragma unroll
            for (int j = 0; j < KCH; ++j) {
                const int t = t0 + (jc + j) * KPP + kin;
                float kf[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) kf[i] = (float)kreg[j][i];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) d = fmaf(qr[g][i], kf[i], d);
#pragma unroll
                    for (int s = LPK / 2; s > 0; s >>= 1) d += __shfl_xor(d, s, WAVE);
                    if (sub == jc + j) sc[g] = (t < nkeys) ? d : -INFINITY;
                }
            }
        }
        // ---- online softmax; lane `lane` now holds key t0 + sub*KPP + kin
        float p[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mnew = fmaxf(m[g], wave_max(sc[g]));    // finite: the block holds at least one real key
            p[g] = __expf(sc[g] - mnew);                        // exp(-inf) = 0 for masked keys
            const float corr = __expf(m[g] - mnew);
            l[g] = l[g] * corr + wave_sum(p[g]);
            m[g] = mnew;
#pragma unroll
            for (int i = 0; i < DPL; ++i) o[g][i] *= corr;
        }
        // ---- weighted values, keys in order; a masked key has probability 0
#pragma unroll
        for (int c = 0; c < WAVE; c += VCH) {
            if (t0 + c < nkeys) {                               // uniform
                VLoad<DPL> vn[VCH];
                if (c + VCH < WAVE && t0 + c + VCH < nkeys) {
#pragma unroll
                    for (int jj = 0; jj < VCH; ++jj) vn[jj].load(vp + (int64_t)min(t0 + c + VCH + jj, nkeys - 1) * kv_stride);
                }
#pragma unroll
                for (int jj = 0; jj < VCH; ++jj) {
                    const int key = c + jj;
                    const int src = (key % KPP) * LPK + key / KPP;      // the lane that holds this key's probability
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const float pj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p[g]), src));
#pragma unroll
                        for (int i = 0; i < DPL; ++i) o[g][i] = fmaf(pj, vr[jj].get(i), o[g][i]);
                    }
                }
#pragma unroll
                for (int jj = 0; jj < VCH; ++jj) vr[jj] = vn[jj];
            }
        }
    }
    // ---- merge the waves (a wave that had no block contributes max = -inf, sum = 0)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (lane == 0) { part_m[wave][g] = m[g]; part_l[wave][g] = l[g]; }
#pragma unroll
        for (int i = 0; i < DPL; ++i) part_o[wave][g][lane * DPL + i] = o[g][i];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < G * HD; e += AD_THREADS) {
        const int g = e / HD, d = e % HD;
        float mx = part_m[0][g];                                // wave 0 always owns block 0
#pragma unroll
        for (int w = 1; w < AD_WAVES; ++w) mx = fmaxf(mx, part_m[w][g]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < AD_WAVES; ++w) {
            const float f = __expf(part_m[w][g] - mx);
            num = fmaf(part_o[w][g][d], f, num);
            den = fmaf(part_l[w][g], f, den);
        }
        const int col = (qh0 + g) * HD + d;
        out[out_tiled ? tiled_off(row, col, (int64_t)hq * HD) : row * (int64_t)hq * HD + col] = (bf16)(num / den);
    }
}

bool attn_decode_supported(int hq, int hkv, int hd) {
    const int g = hkv > 0 ? hq / hkv : 0;
    return (hd == 64 || hd == 128) && hq == g * hkv && (g == 1 || g == 2 || g == 4 || g == 8);
}

template <int G>
static void launch_g(const bf16* q, int64_t q_stride, const bf16* k, const bf16* v, int64_t kv_stride, const int32_t* kv_row0,
                     const int32_t* npos, bf16* out, int64_t rows, int hq, int hkv, int hd, hipStream_t s, bool out_tiled) {
    const float scale = 1.0f / sqrtf((float)hd);
    dim3 grid((unsigned)rows, (unsigned)(hq / G));
    if (hd == 64)
        attn_decode_kernel<G, 64><<<grid, AD_THREADS, 0, s>>>(q, q_stride, k, v, kv_stride, kv_row0, npos, out, hq, hq / hkv, scale, out_tiled);
    else
        attn_decode_kernel<G, 128><<<grid, AD_THREADS, 0, s>>>(q, q_stride, k, v, kv_stride, kv_row0, npos, out, hq, hq / hkv, scale, out_tiled);
}

void launch_attn_decode(const void* q, int64_t q_stride, const void* k, const void* v, int64_t kv_stride,
                        const int32_t* kv_row0, const int32_t* npos, void* out, int64_t rows, int hq, int hkv, int hd,
                        hipStream_t s, bool out_tiled) {
    if (rows <= 0) return;
    const bf16 *qq = (const bf16*)q, *kk = (const bf16*)k, *vv = (const bf16*)v;
    int g = hq / hkv;                                           // heads per workgroup: halve until the grid covers the chip
    while (g > 1 && rows * (hq / g) < AD_FILL) g >>= 1;
    switch (g) {
        case 1: launch_g<1>(qq, q_stride, kk, vv, kv_stride, kv_row0, npos, (bf16*)out, rows, hq, hkv, hd, s, out_tiled); break;
        case 2: launch_g<2>(qq, q_stride, kk, vv, kv_stride, kv_row0, npos, (bf16*)out, rows, hq, hkv, hd, s, out_tiled); break;
        case 4: launch_g<4>(qq, q_stride, kk, vv, kv_stride, kv_row0, npos, (bf16*)out, rows, hq, hkv, hd, s, out_tiled); break;
        default: launch_g<8>(qq, q_stride, kk, vv, kv_stride, kv_row0, npos, (bf16*)out, rows, hq, hkv, hd, s, out_tiled); break;
    }
}

}  // namespace vl
