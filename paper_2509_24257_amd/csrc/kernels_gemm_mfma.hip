// C[M,N] = A[M,K] * W[N,K]^T in bf16 on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
// Both operands are K-contiguous, so every global load, LDS write and LDS read moves 16-byte vectors of 8
// consecutive k values - exactly what one lane feeds to the MFMA.
//
//   workgroup : 512 lanes = 8 waves, output tile 256 x 256, K stepped by 32
//   waves     : two groups of four (one wave of each group on every SIMD); group g owns rows 128 g .. 128 g + 127,
//               wave w of a group owns columns 64 w .. 64 w + 63 as 4 x 2 MFMA blocks of 32x32 (128 accumulator
//               VGPRs)
//   ping-pong : both groups run the same stream, [memory phase | barrier | compute phase | barrier] per k-tile,
//               but group 1 runs one phase behind group 0 (it takes one extra barrier before the loop, group 0 one
//               after it).  While one wave of a SIMD issues its 16 MFMAs the other one does its LDS reads and
//               global loads, so the matrix pipe is handed from wave to wave instead of idling.
//   LDS       : a ring of 5 slots of 32 KB (= all 160 KB of the CU), slot = (256 + 256) rows x 32 k.  Rows are 64 B,
//               unpadded; the four 16-byte chunks of row r are XOR-swizzled by (r / 4) % 4 so that the 16 lanes the
//               LDS serves per clock always hit 16 different 16-byte bank groups (measured: zero bank conflicts).
//   loads     : global -> LDS directly (global_load_lds_dwordx4, no staging registers).  One such instruction
//               fills 1 KB = 16 consecutive LDS rows; the swizzle is applied on the global-address side.  The loads
//               of tile p+4 are issued in the memory phase of tile p into the slot tile p-1 has just left, so every
//               load has three tile periods to land; "vmcnt(12)" before the barrier of that phase guarantees this
//               wave's part of tile p+1 is in LDS before anybody reads it.
//   persistent: one workgroup per CU walks several output tiles; the first four k-tiles of the next tile are requested
//               before the epilogue of the current one, so they land while the results are written out
//   placement : workgroup ids are dealt round-robin to the 8 XCDs, so ids are remapped such that each XCD walks its
//               own contiguous run of tiles, 8 M-tiles deep before moving to the next N-tile; the 32 tiles an XCD has
//               in flight then share A and W panels through that XCD's L2.
//   MFMA layout (32x32x16): operand lane l carries row (l % 32) and 8 consecutive k of half (l / 32);
//               result register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l % 32].
//
// Epilogues: store as bf16 / store as fp32 / add into the fp32 residual stream / SwiGLU on interleaved gate|up
// column blocks (W rows alternate 32 gate rows and 32 up rows, so MFMA block j=0 is gate and j=1 is up of the same
// 32 channels and the product silu(gate)*up never leaves registers) / column-wise argmax (the LM head run with the
// vocabulary as rows: a lane's 64 accumulators of a column are 64 logits of one token, so each wave reduces its
// 128 x 64 block to a maximum and its lowest index per token in registers, plus one exchange between the lane halves).
#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int GM_BM = 256, GM_BN = 256, GM_BK = 32;
constexpr int GM_ROWB = 64;                                     // bytes per LDS row (32 bf16)
constexpr int GM_OPER = 256 * GM_ROWB;                          // 16 KB per operand per slot
constexpr int GM_SLOT = 2 * GM_OPER;                            // 32 KB
constexpr int GM_SLOTS = 5;                                     // 160 KB: the whole LDS of a CU
constexpr int GM_THREADS = 512;
constexpr int GM_GROUP_M = 8;
constexpr int GM_XCDS = 8;

#define GM_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define GM_GLB(p) ((const __attribute__((address_space(1))) void*)(p))
// s_barrier fenced for the instruction scheduler: nothing moves across a phase boundary
#define GM_BARRIER() do { __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_barrier(); __builtin_amdgcn_sched_barrier(0); } while (0)
// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
constexpr int GM_WAIT_VM12_LGKM0 = 0x007C;                      // vmcnt(12) lgkmcnt(0)
constexpr int GM_WAIT_VM0_LGKM0 = 0x0070;                       // vmcnt(0)  lgkmcnt(0)

template <int EPI>
__global__ __launch_bounds__(GM_THREADS, 1) void gemm_mfma_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                                                                  int M, int N, int K, void* __restrict__ outp,
                                                                  int tiles_m, int tiles_n, int layout, ArgmaxParts ap) {
    __shared__ __align__(1024) unsigned char ring[GM_SLOTS * GM_SLOT];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = wave >> 2, wn = wave & 3;

    // ---- XCD-aware tile order.  Workgroup ids are dealt round-robin to the XCDs; this workgroup walks the virtual
    // ids blockIdx.x, + gridDim.x, ... (gridDim.x is a multiple of 8, so all of them land on its own XCD), and virtual
    // id v is tile (v % 8) * per_xcd + v / 8 of the XCD-major order.
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + GM_XCDS - 1) / GM_XCDS;
    const int n_virtual = per_xcd * GM_XCDS;
    auto tile_of = [&](int v, int& m0, int& n0) -> bool {       // uniform for the whole workgroup
        if (v >= n_virtual) return false;
        const int pid = (v % GM_XCDS) * per_xcd + (v / GM_XCDS);
        if (pid >= total) return false;                         // only the last ids of the last XCD: nothing follows
        const int group_span = GM_GROUP_M * tiles_n;
        const int group = pid / group_span;
        const int first_m = group * GM_GROUP_M;
        const int gsize = min(tiles_m - first_m, GM_GROUP_M);
        const int in_group = pid - group * group_span;
        m0 = (first_m + in_group % gsize) * GM_BM;
        n0 = (in_group / gsize) * GM_BN;
        return true;
    };

    // ---- direct-to-LDS sources.  Load i (0,1) of this wave fills LDS rows 16*(wave + 8 i) .. +15 of an operand:
    // lane -> (row = 16*(wave + 8 i) + lane/4, physical chunk = lane%4), which must hold logical chunk
    // phys ^ ((row/4)%4).  Rows past the matrix edge re-read the last row (their results are never stored).
    // A tiled operand (see tiled_off) is padded to whole 256-row blocks and its k-tiles are 16 KB apart.
    const bf16* ga[2];
    const bf16* gw[2];
    const int a_step = (layout & GL_A_TILED) ? TL_PIECE : GM_BK;        // elements between consecutive k-tiles
    const int w_step = (layout & GL_W_TILED) ? TL_PIECE : GM_BK;
    auto point_at = [&](int m0, int n0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = 16 * (wave + 8 * i) + (lane >> 2);
            const int c = (lane & 3) ^ ((row >> 2) & 3);
            ga[i] = (layout & GL_A_TILED) ? A + tiled_off(m0 + row, 0, K) + c * 8 : A + (int64_t)min(m0 + row, M - 1) * K + c * 8;
            gw[i] = (layout & GL_W_TILED) ? W + tiled_off(n0 + row, 0, K) + c * 8 : W + (int64_t)min(n0 + row, N - 1) * K + c * 8;
        }
    };
    const int dma_off = wave * 1024;                            // + i * 8192, + GM_OPER for W

    // ---- MFMA operand reads: lane (row fr, half fh) reads logical chunk 2s + fh of rows fr + 32 i
    const int fr = lane & 31, fh = lane >> 5;
    const int sw = (fr >> 2) & 3;                               // (row/4)%4 is the same for rows fr + 32 i
    int a_off[2], w_off[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int phys = (2 * s + fh) ^ sw;
        a_off[s] = (grp * 128 + fr) * GM_ROWB + phys * 16;
        w_off[s] = GM_OPER + (wn * 64 + fr) * GM_ROWB + phys * 16;
    }
    const int KT = K / GM_BK;
    const int col_in = lane & 31, row_half = (lane >> 5) * 4;   // epilogue: lane l of a 32x32 block holds column l%32

#define GM_DMA_TILE(SLOT, KTILE)                                                                              \
    {                                                                                                         \
        unsigned char* dst_ = ring + (SLOT) * GM_SLOT + dma_off;                                              \
        __builtin_amdgcn_global_load_lds(GM_GLB(ga[0] + (int64_t)(KTILE) * a_step), GM_LDS(dst_), 16, 0, 0);  \
        __builtin_amdgcn_global_load_lds(GM_GLB(gw[0] + (int64_t)(KTILE) * w_step), GM_LDS(dst_ + GM_OPER), 16, 0, 0); \
        __builtin_amdgcn_global_load_lds(GM_GLB(ga[1] + (int64_t)(KTILE) * a_step), GM_LDS(dst_ + 8192), 16, 0, 0); \
        __builtin_amdgcn_global_load_lds(GM_GLB(gw[1] + (int64_t)(KTILE) * w_step), GM_LDS(dst_ + GM_OPER + 8192), 16, 0, 0); \
    }
    // k-tiles 0 .. 3 of the tile `ga`/`gw` point at, into slots 0 .. 3
#define GM_PROLOGUE()                                                                                         \
    _Pragma("unroll") for (int p_ = 0; p_ < GM_SLOTS - 1; ++p_)                                               \
        if (p_ < KT) GM_DMA_TILE(p_, p_)

    int v = blockIdx.x, m0 = 0, n0 = 0;
    if (!tile_of(v, m0, n0)) return;
    point_at(m0, n0);
    GM_PROLOGUE()

    // ---- one output tile per iteration.  The first loads of the NEXT tile are issued before the epilogue of this one,
    // so they land while the results are written out.
    for (;;) {
        f32x16 acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // everything issued so far (the prologue loads, the previous tile's stores) has completed; publish
        __builtin_amdgcn_s_waitcnt(GM_WAIT_VM0_LGKM0);
        GM_BARRIER();
        if (grp == 1) GM_BARRIER();                             // group 1 runs one phase behind group 0

        bf16x8 af[2][4], wf[2][2];
        int slot_rd = 0, slot_wr = GM_SLOTS - 1;
        for (int p = 0; p < KT; ++p) {
            // ---- memory phase: MFMA operands of tile p
            const unsigned char* base = ring + slot_rd * GM_SLOT;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int i = 0; i < 4; ++i) af[s][i] = *(const bf16x8*)(base + a_off[s] + i * 32 * GM_ROWB);
#pragma unroll
                for (int j = 0; j < 2; ++j) wf[s][j] = *(const bf16x8*)(base + w_off[s] + j * 32 * GM_ROWB);
            }
            // the loads of tile p+4 go out while those reads are in flight; their slot held tile p-1, which the other
            // group finished reading before the barrier that ended its previous memory phase
            const bool more = p + GM_SLOTS - 1 < KT;
            if (more) GM_DMA_TILE(slot_wr, p + GM_SLOTS - 1)
            // this wave has issued tiles <= p+4, four loads each: at most three tiles may remain in flight, so that
            // its part of tile p+1 has landed before the barrier below publishes it
            if (more) __builtin_amdgcn_s_waitcnt(GM_WAIT_VM12_LGKM0);
            else __builtin_amdgcn_s_waitcnt(GM_WAIT_VM0_LGKM0);
            GM_BARRIER();
            // ---- compute phase (raised priority: the MFMAs win issue arbitration over the other wave's memory phase)
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s][i], wf[s][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
            GM_BARRIER();
            slot_rd = slot_rd + 1 == GM_SLOTS ? 0 : slot_rd + 1;
            slot_wr = slot_wr + 1 == GM_SLOTS ? 0 : slot_wr + 1;
        }
        if (grp == 0) GM_BARRIER();                             // every wave has passed the same number of barriers

        // ---- every wave has finished reading the ring: start on the next tile's first k-tiles
        const int cm0 = m0, cn0 = n0;
        v += gridDim.x;
        const bool next = tile_of(v, m0, n0);
        if (next) {
            point_at(m0, n0);
            GM_PROLOGUE()
        }

        // ---- epilogue of tile (cm0, cn0).  Lane l of a 32x32 block holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4.
        const bool interior = (cm0 + GM_BM <= M) && (cn0 + GM_BN <= N);    // uniform: no per-element guards needed
        if (EPI == EPI_ARGMAX) {
            const int part = (cm0 >> 7) + grp;                  // this wave's 128 rows
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = cn0 + wn * 64 + j * 32 + col_in;
                const int want = (ap.tok && col < N) ? ap.tok[col] : -1;
                float bv = -INFINITY, zt = 0.f;
                int bi = 0x7fffffff;
                bool hit = false;
                // rows in ascending order within the lane: strict '>' keeps the lowest index among equals; NaN never wins
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = cm0 + grp * 128 + i * 32 + (r >> 2) * 8 + row_half + (r & 3);
                        const float v = acc[i][j][r];
                        if (row < M) {
                            if (v > bv) { bv = v; bi = row; }
                            if (row == want) { zt = v; hit = true; }
                        }
                    }
                const float ov = __shfl_xor(bv, 32, WAVE);      // the other half of the rows
                const int oi = __shfl_xor(bi, 32, WAVE);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                if (col < N && cm0 + grp * 128 < M) {           // (a wave whose rows all lie past the matrix has no part)
                    if (lane < 32) {
                        ap.pmax[part * ap.ld + col] = bv;
                        ap.pidx[part * ap.ld + col] = bi;
                    }
                    if (hit) ap.ztok[col] = zt;
                }
            }
        } else if (interior) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int mb = cm0 + grp * 128 + i * 32 + row_half;
                if (EPI == EPI_SWIGLU) {
                    const int F = N >> 1;
                    const int f = ((cn0 + wn * 64) >> 1) + col_in;
                    // row-major: rows F apart; tiled: the 32 channels of this block sit in one piece, rows 32 elements apart
                    bf16* out = (bf16*)outp + ((layout & GL_OUT_TILED) ? tiled_off(mb, f, F) : (int64_t)mb * F + f);
                    const int64_t rs = (layout & GL_OUT_TILED) ? TL_K : F;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float g = acc[i][0][r], u = acc[i][1][r];
                        out[(int64_t)((r >> 2) * 8 + (r & 3)) * rs] = (bf16)silu_mul(g, u);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int64_t base = (int64_t)mb * N + cn0 + wn * 64 + j * 32 + col_in;
                        if (EPI == EPI_ADD_RESID) {
                            // all sixteen residual loads of a block go out before the first one is needed
                            float* out = (float*)outp + base;
                            float old[16];
#pragma unroll
                            for (int r = 0; r < 16; ++r) old[r] = out[(int64_t)((r >> 2) * 8 + (r & 3)) * N];
#pragma unroll
                            for (int r = 0; r < 16; ++r) out[(int64_t)((r >> 2) * 8 + (r & 3)) * N] = old[r] + acc[i][j][r];
                        } else if (EPI == EPI_STORE_F32) {
                            float* out = (float*)outp + base;
#pragma unroll
                            for (int r = 0; r < 16; ++r) out[(int64_t)((r >> 2) * 8 + (r & 3)) * N] = acc[i][j][r];
                        } else {
                            bf16* out = (bf16*)outp + base;
#pragma unroll
                            for (int r = 0; r < 16; ++r) out[(int64_t)((r >> 2) * 8 + (r & 3)) * N] = (bf16)acc[i][j][r];
                        }
                    }
                }
            }
        } else {
            // edge tiles: the same stores with row and column guards
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int mb = cm0 + grp * 128 + i * 32 + row_half;
                if (EPI == EPI_SWIGLU) {
                    const int F = N >> 1;
                    bf16* out = (bf16*)outp;
                    const int f = ((cn0 + wn * 64) >> 1) + col_in;
                    if (f < F) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int m = mb + (r >> 2) * 8 + (r & 3);
                            if (m < M) {
                                const float g = acc[i][0][r], u = acc[i][1][r];
                                out[(layout & GL_OUT_TILED) ? tiled_off(m, f, F) : (int64_t)m * F + f] = (bf16)silu_mul(g, u);
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int n = cn0 + wn * 64 + j * 32 + col_in;
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
        if (!next) break;
    }
#undef GM_PROLOGUE
#undef GM_DMA_TILE
}

// One workgroup per compute unit (a workgroup takes all 160 KB of a CU's LDS anyway), each walking several tiles.
static int resident_workgroups() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < GM_XCDS)
            cus = 256;
        n = cus / GM_XCDS * GM_XCDS;
    }
    return n;
}

template <int EPI>
static void launch_one(const bf16* A, const bf16* W, int M, int N, int K, void* out, hipStream_t s, int layout) {
    const int tiles_m = (M + GM_BM - 1) / GM_BM, tiles_n = (N + GM_BN - 1) / GM_BN;
    const int total = tiles_m * tiles_n;
    const int grid = std::min(((total + GM_XCDS - 1) / GM_XCDS) * GM_XCDS, resident_workgroups());
    gemm_mfma_kernel<EPI><<<dim3((unsigned)grid), GM_THREADS, 0, s>>>(A, W, M, N, K, out, tiles_m, tiles_n, layout, ArgmaxParts{});
}

void launch_gemm_mfma(const void* A, const void* W, int M, int N, int K, int epi, void* out, hipStream_t s, int layout) {
    if (M <= 0 || N <= 0) return;
    const bf16* a = (const bf16*)A;
    const bf16* w = (const bf16*)W;
    switch (epi) {
        case EPI_STORE: launch_one<EPI_STORE>(a, w, M, N, K, out, s, layout); break;
        case EPI_STORE_F32: launch_one<EPI_STORE_F32>(a, w, M, N, K, out, s, layout); break;
        case EPI_ADD_RESID: launch_one<EPI_ADD_RESID>(a, w, M, N, K, out, s, layout); break;
        default: launch_one<EPI_SWIGLU>(a, w, M, N, K, out, s, layout); break;
    }
}

void launch_gemm_mfma_argmax(const void* X, const void* Wlm, int tokens, int vocab, int K, const ArgmaxParts& parts, hipStream_t s,
                             int layout) {
    if (tokens <= 0 || vocab <= 0) return;
    // transposed: the vocabulary is the row operand, the tokens are the column operand
    const int M = vocab, N = tokens;
    const int lay = ((layout & GL_W_TILED) ? GL_A_TILED : 0) | ((layout & GL_A_TILED) ? GL_W_TILED : 0);
    const int tiles_m = (M + GM_BM - 1) / GM_BM, tiles_n = (N + GM_BN - 1) / GM_BN;
    const int total = tiles_m * tiles_n;
    const int grid = std::min(((total + GM_XCDS - 1) / GM_XCDS) * GM_XCDS, resident_workgroups());
    gemm_mfma_kernel<EPI_ARGMAX><<<dim3((unsigned)grid), GM_THREADS, 0, s>>>((const bf16*)Wlm, (const bf16*)X, M, N, K, nullptr, tiles_m,
                                                                             tiles_n, lay, parts);
}

}  // namespace vl
