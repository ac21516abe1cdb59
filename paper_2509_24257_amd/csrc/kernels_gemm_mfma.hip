// C[M,N] = A[M,K] * W[N,K]^T in bf16 on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
// Both operands are K-contiguous, so every global load, LDS store and LDS load is a 16-byte vector of 8
// consecutive k values - exactly what one lane feeds to the MFMA.
//
//   workgroup : 512 lanes = 8 waves, output tile 256 x 256, K stepped by 64
//   waves     : 2 (M) x 4 (N); each wave owns 128 x 64 = 4 x 2 MFMA blocks of 32x32 -> 128 accumulator VGPRs
//   LDS       : two stages of (256 + 256) rows x 64 k, row pitch 72 elements (144 B): the 16-byte pad makes
//               consecutive rows land on different banks for the MFMA operand reads; 144 KB of the CU's 160 KB
//   pipeline  : the loads of k-tile t+1 are issued into registers before the MFMAs of tile t and written to
//               the other LDS stage after them; one barrier per k-tile
//   placement : workgroup ids are dealt round-robin to the 8 XCDs, so ids are remapped such that each XCD
//               walks its own contiguous run of tiles, 8 M-tiles deep before moving to the next N-tile;
//               the 32 tiles an XCD has in flight then share A and W panels through that XCD's L2
//   MFMA layout (32x32x16): operand lane l carries row (l % 32) and 8 consecutive k of half (l / 32);
//               result register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l % 32]
#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int GM_BM = 256, GM_BN = 256, GM_BK = 64;
constexpr int GM_PITCH = 72;                                // elements per LDS row
constexpr int GM_THREADS = 512;
constexpr int GM_STAGE = (GM_BM + GM_BN) * GM_PITCH;        // elements per stage
constexpr int GM_LDS_BYTES = 2 * GM_STAGE * 2;
constexpr int GM_GROUP_M = 8;
constexpr int GM_XCDS = 8;

template <int EPI>
__global__ __launch_bounds__(GM_THREADS, 1) void gemm_mfma_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                                                                  int M, int N, int K, void* __restrict__ outp,
                                                                  int tiles_m, int tiles_n) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16* lds = (bf16*)smem_raw;

    // ---- XCD-aware tile order
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + GM_XCDS - 1) / GM_XCDS;
    const int pid = (blockIdx.x % GM_XCDS) * per_xcd + (blockIdx.x / GM_XCDS);
    if (pid >= total) return;                               // uniform for the whole workgroup
    const int group_span = GM_GROUP_M * tiles_n;
    const int group = pid / group_span;
    const int first_m = group * GM_GROUP_M;
    const int gsize = min(tiles_m - first_m, GM_GROUP_M);
    const int in_group = pid - group * group_span;
    const int tm = first_m + in_group % gsize;
    const int tn = in_group / gsize;
    const int m0 = tm * GM_BM, n0 = tn * GM_BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;

    // ---- global -> LDS staging: lane handles 16-byte chunk (row = id / 8, chunk = id % 8), 4 of A and 4 of W
    const bf16* ga[4];
    const bf16* gw[4];
    int lds_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + GM_THREADS * i;
        const int row = id >> 3, c = id & 7;
        ga[i] = A + (int64_t)min(m0 + row, M - 1) * K + c * 8;      // rows past the edge re-read the last row
        gw[i] = W + (int64_t)min(n0 + row, N - 1) * K + c * 8;
        lds_off[i] = row * GM_PITCH + c * 8;
    }
    uint4 ra[4], rw[4];
    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ra[i] = *(const uint4*)(ga[i] + kt * GM_BK);
            rw[i] = *(const uint4*)(gw[i] + kt * GM_BK);
        }
    };
    auto lstore = [&](int stage) {
        bf16* as = lds + stage * GM_STAGE;
        bf16* ws = as + GM_BM * GM_PITCH;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(uint4*)(as + lds_off[i]) = ra[i];
            *(uint4*)(ws + lds_off[i]) = rw[i];
        }
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int frag_row = lane & 31, frag_half = lane >> 5;
    const int a_base = (wm * 128 + frag_row) * GM_PITCH + frag_half * 8;
    const int w_base = (wn * 64 + frag_row) * GM_PITCH + frag_half * 8;

    const int KT = K / GM_BK;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) gload(kt + 1);
        const bf16* as = lds + cur * GM_STAGE;
        const bf16* ws = as + GM_BM * GM_PITCH;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 af[4], wf[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *(const bf16x8*)(as + a_base + i * 32 * GM_PITCH + s * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j) wf[j] = *(const bf16x8*)(ws + w_base + j * 32 * GM_PITCH + s * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  Lane l of a 32x32 block holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4.
    const int col_in = lane & 31, row_half = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int mb = m0 + wm * 128 + i * 32 + row_half;
        if (EPI == EPI_SWIGLU) {
            // W rows alternate 32 gate rows / 32 up rows, so block j=0 is gate and j=1 is up of the same 32 channels
            const int F = N >> 1;
            const int f = ((n0 + wn * 64) >> 1) + col_in;
            bf16* out = (bf16*)outp;
            if (f < F) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mb + (r >> 2) * 8 + (r & 3);
                    if (m < M) {
                        const float g = acc[i][0][r], u = acc[i][1][r];
                        out[(int64_t)m * F + f] = (bf16)(g / (1.0f + __expf(-g)) * u);
                    }
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + col_in;
                if (n >= N) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mb + (r >> 2) * 8 + (r & 3);
                    if (m >= M) continue;
                    const int64_t o = (int64_t)m * N + n;
                    if (EPI == EPI_STORE) ((bf16*)outp)[o] = (bf16)acc[i][j][r];
                    if (EPI == EPI_STORE_F32) ((float*)outp)[o] = acc[i][j][r];
                    if (EPI == EPI_ADD_RESID) ((float*)outp)[o] += acc[i][j][r];
                }
            }
        }
    }
}

template <int EPI>
static void launch_one(const bf16* A, const bf16* W, int M, int N, int K, void* out, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, GM_LDS_BYTES);
        attr_set = true;
    }
    const int tiles_m = (M + GM_BM - 1) / GM_BM, tiles_n = (N + GM_BN - 1) / GM_BN;
    const int total = tiles_m * tiles_n;
    const int grid = ((total + GM_XCDS - 1) / GM_XCDS) * GM_XCDS;
    gemm_mfma_kernel<EPI><<<dim3((unsigned)grid), GM_THREADS, GM_LDS_BYTES, s>>>(A, W, M, N, K, out, tiles_m, tiles_n);
}

void launch_gemm_mfma(const void* A, const void* W, int M, int N, int K, int epi, void* out, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    const bf16* a = (const bf16*)A;
    const bf16* w = (const bf16*)W;
    switch (epi) {
        case EPI_STORE: launch_one<EPI_STORE>(a, w, M, N, K, out, s); break;
        case EPI_STORE_F32: launch_one<EPI_STORE_F32>(a, w, M, N, K, out, s); break;
        case EPI_ADD_RESID: launch_one<EPI_ADD_RESID>(a, w, M, N, K, out, s); break;
        default: launch_one<EPI_SWIGLU>(a, w, M, N, K, out, s); break;
    }
}

}  // namespace vl
