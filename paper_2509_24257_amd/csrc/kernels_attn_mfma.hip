// Causal grouped-query flash attention for the bf16 prefill, on the gfx950 matrix cores.
//
// One workgroup (4 waves) handles 128 consecutive queries of one sequence for one query head; each wave owns
// 32 queries.  Keys are walked 64 at a time; the K tile [64 keys][hd] and the transposed V tile [hd][64 keys]
// are staged in LDS (rows padded by 16 bytes so that the MFMA operand reads of consecutive rows hit
// different banks).  Everything is computed TRANSPOSED so that one lane always owns one query:
//
//   S^T[key][q] = K * Q^T      A operand = K rows from LDS, B operand = Q rows held in registers
//   O^T[c][q]  += V^T * P^T    A operand = V^T rows from LDS, B operand = P^T straight from the S^T registers
//
// With the 32x32x16 MFMA the result lane l holds column (l % 32) = the query, and its 16 registers hold rows
// 8*(r/4) + 4*(l/32) + r%4 = keys (or channels).  The running max / sum / rescale of the online softmax are
// therefore per-lane scalars, and the row reductions are over a lane's own registers plus one exchange with
// lane l^32.  The probabilities feed the second MFMA without leaving registers: the k index of that MFMA is
// a dummy (contraction) index, so any assignment of keys to (register, lane half) is valid as long as the
// V^T operand is gathered with the same assignment - two 8-byte LDS reads per operand.
//
// Softmax statistics and all accumulators are fp32; probabilities are rounded to bf16 for the second MFMA.
#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int FA_BQ = 128;        // queries per workgroup
constexpr int FA_BK = 64;         // keys per step
constexpr int FA_THREADS = 256;

template <int HD>
__global__ __launch_bounds__(FA_THREADS, 2) void attn_mfma_kernel(const bf16* __restrict__ qkv, int64_t n_rows,
                                                               const bf16* __restrict__ vt, int64_t ldv,
                                                               const AttnTile* __restrict__ tiles,
                                                               bf16* __restrict__ out, int hq, int hkv, float scale_log2e,
                                                               bool out_tiled) {
    constexpr int KP = HD + 8;               // K tile row pitch (elements)
    constexpr int VP = FA_BK + 8;            // V^T tile row pitch
    constexpr int KSTEPS = HD / 16;          // MFMA k-steps over the head dimension
    constexpr int DB = HD / 32;              // 32-channel output blocks
    __shared__ __align__(16) bf16 ks[FA_BK * KP];
    __shared__ __align__(16) bf16 vs[HD * VP];

    const AttnTile t = tiles[blockIdx.x];
    const int head = blockIdx.y, g = head / (hq / hkv);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, half = lane >> 5;
    const int64_t pitch = (int64_t)(hq + 2 * hkv) * HD;

    // ---- this lane's query row (clamped into the tile; rows past q_rows are computed and dropped)
    const int q_local = wave * 32 + lq;
    const int q_idx = min(q_local, t.q_rows - 1);
    const int q_pos = t.pos0 + q_idx;
    const bf16* qp = qkv + (int64_t)(t.q_row0 + q_idx) * pitch + (int64_t)head * HD + half * 8;
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *(const bf16x8*)(qp + s * 16);

    f32x16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;      // l_run: this lane half's share of the row sum

    const bf16* kbase = qkv + (int64_t)hq * HD + (int64_t)g * HD;
    const bf16* vbase = vt + (int64_t)g * HD * ldv + t.vt_col0;
    const int n_kv_tiles = (t.kv_len + FA_BK - 1) / FA_BK;
    const int wave_first_pos = t.pos0 + wave * 32;

    // The tiles travel global -> registers -> LDS; the registers of tile kt+1 are requested right after tile kt has been
    // published in LDS, so the memory latency runs behind the arithmetic of tile kt.
    constexpr int KLD = (FA_BK * HD / 8) / FA_THREADS, VLD = (HD * FA_BK / 8) / FA_THREADS;
    u32x4 kreg[KLD], vreg[VLD];
    auto fetch = [&](int key0) {
        // K tile: 64 rows x HD, 16-byte chunks; rows past the end of the buffer re-read the last row (masked below)
#pragma unroll
        for (int i = 0; i < KLD; ++i) {
            const int id = tid + FA_THREADS * i;
            const int row = id / (HD / 8), c = id % (HD / 8);
            const int64_t grow = min((int64_t)t.kv_row0 + key0 + row, n_rows - 1);
            kreg[i] = *(const u32x4*)(kbase + grow * pitch + c * 8);
        }
        // V^T tile: HD rows x 64 keys (the vt buffer is padded, so the columns always exist)
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int id = tid + FA_THREADS * i;
            const int row = id >> 3, c = id & 7;
            vreg[i] = *(const u32x4*)(vbase + (int64_t)row * ldv + key0 + c * 8);
        }
    };
    fetch(0);
    const int wave_last_pos = t.pos0 + min(wave * 32 + 31, t.q_rows - 1);

    for (int kt = 0; kt < n_kv_tiles; ++kt) {
        const int key0 = kt * FA_BK;
        __syncthreads();                                         // everyone is done with the previous tiles
#pragma unroll
        for (int i = 0; i < KLD; ++i) {
            const int id = tid + FA_THREADS * i;
            *(u32x4*)(ks + (id / (HD / 8)) * KP + (id % (HD / 8)) * 8) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int id = tid + FA_THREADS * i;
            *(u32x4*)(vs + (id >> 3) * VP + (id & 7) * 8) = vreg[i];
        }
        __syncthreads();
        if (kt + 1 < n_kv_tiles) fetch(key0 + FA_BK);
        if (key0 > wave_last_pos) continue;                      // uniform per wave: every key of the tile is masked

        // ---- S^T = K Q^T for the two 32-key blocks of this tile
        f32x16 st[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) st[kb][r] = 0.f;
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const bf16x8 kf = *(const bf16x8*)(ks + (kb * 32 + lq) * KP + s * 16 + half * 8);
                st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], st[kb], 0, 0, 0);
            }
        }
        // ---- scale (to base-2 logits), causal mask, running max
        const bool need_mask = key0 + FA_BK - 1 > wave_first_pos;     // uniform per wave
        float m_new = m_run;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = st[kb][r] * scale_log2e;
                if (need_mask) {
                    const int key = key0 + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                    if (key > q_pos) v = -INFINITY;
                }
                st[kb][r] = v;
                m_new = fmaxf(m_new, v);
            }
        m_new = fmaxf(m_new, __shfl_xor(m_new, 32, WAVE));           // key 0 is visible to every query: finite
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(st[kb][r] - m_new);
                st[kb][r] = p;
                psum += p;
            }
        l_run = l_run * corr + psum;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[b][r] *= corr;

        // ---- O^T += V^T P^T.  MFMA step (kb, s2) contracts over the 16 keys held in registers 8*s2 .. 8*s2+7
        // of both lane halves: keys kb*32 + 16*s2 + {4*half .. +3} and {8 + 4*half .. +3}.
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (bf16)st[kb][8 * s2 + e];
                const int kcol = kb * 32 + s2 * 16 + half * 4;
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    const bf16* vr = vs + (b * 32 + lq) * VP + kcol;
                    const bf16x4 lo = *(const bf16x4*)vr;
                    const bf16x4 hi = *(const bf16x4*)(vr + 8);
                    bf16x8 vf;
                    vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
                    vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
                    o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[b], 0, 0, 0);
                }
            }
    }

    // ---- normalise and store: lane holds query q_local, channels b*32 + 8*(r/4) + 4*half + r%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, WAVE);
    const float inv = 1.0f / l_tot;
    if (q_local < t.q_rows) {
        const int64_t orow = t.q_row0 + q_local;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[b][rg * 4 + e] * inv);
                const int col = head * HD + b * 32 + rg * 8 + half * 4;            // 4 | 32: never straddles a piece
                *(bf16x4*)(out + (out_tiled ? tiled_off(orow, col, (int64_t)hq * HD) : orow * hq * HD + col)) = v;
            }
    }
}

void launch_attn_mfma(const void* qkv, int64_t n_rows, const void* vt, int64_t ldv, const AttnTile* tiles, int n_tiles,
                      void* out, int hq, int hkv, int hd, hipStream_t s, bool out_tiled) {
    if (n_tiles <= 0) return;
    const float scale_log2e = (1.0f / sqrtf((float)hd)) * 1.4426950408889634f;
    dim3 grid((unsigned)n_tiles, (unsigned)hq);
    if (hd == 128)
        attn_mfma_kernel<128><<<grid, FA_THREADS, 0, s>>>((const bf16*)qkv, n_rows, (const bf16*)vt, ldv, tiles, (bf16*)out, hq,
                                                          hkv, scale_log2e, out_tiled);
    else
        attn_mfma_kernel<64><<<grid, FA_THREADS, 0, s>>>((const bf16*)qkv, n_rows, (const bf16*)vt, ldv, tiles, (bf16*)out, hq,
                                                         hkv, scale_log2e, out_tiled);
}

}  // namespace vl
