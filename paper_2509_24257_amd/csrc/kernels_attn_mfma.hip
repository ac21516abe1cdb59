// Causal grouped-query flash attention for the bf16 prefill, on the gfx950 matrix cores.
//
// One workgroup = 4 waves, one per SIMD, each with up to 512 registers.  A wave owns 64 queries of one query head
// (two MFMA column blocks of 32), so every key / value fragment it reads from LDS feeds two MFMAs.  The four waves of
// a workgroup always share one KV head and therefore one stream of key / value tiles:
//   HPW = 4 : four query heads of the group x the same 64 queries          (Hq / Hkv a multiple of 4)
//   HPW = 2 : two query heads x two consecutive 64-query sub-tiles          (Hq / Hkv even)
//   HPW = 1 : one query head x four consecutive 64-query sub-tiles          (otherwise)
//
// Everything is computed TRANSPOSED so that one lane always owns one query:
//   S^T[key][q] = K * Q^T      A operand = K rows from LDS, B operand = Q rows held in registers
//   O^T[c][q]  += V^T * P^T    A operand = V^T rows from LDS, B operand = P^T straight from the S^T registers
// With the 32x32x16 MFMA the result lane l holds column (l % 32) = the query, and its 16 registers hold rows
// 8*(r/4) + 4*(l/32) + r%4.  The K fragment puts key perm(i) on row i, perm swapping bits 2 and 3 of i; register r
// of lane half h then holds key 16*(r/8) + 8*h + r%8 of the 32-key block, so registers 8*s2 .. 8*s2+7 are eight
// CONSECUTIVE keys - exactly one 16-byte read of a V^T row for the second MFMA, whose contraction index they become.
//
// Keys are walked in blocks of 32 inside tiles of 64.  Tiles travel global -> LDS directly (buffer loads that write
// LDS, 16 bytes per lane) into a ring of four slots; the 16-byte chunks of a row are XOR-swizzled on the global-address
// side so the fragment reads are free of bank conflicts.  One barrier per tile; the loads of the tile after next are
// spread over the slots of the tile's first step.
//
// Software pipeline over blocks j: while the vector ALUs turn S_j into probabilities P_j, the matrix pipe computes
// S_{j+1} and O += V_{j-1} P_{j-1}.  No MFMA of a step depends on a vector result of the same step.  Q sits in AGPRs and
// feeds the first MFMA directly, S is produced in VGPRs (those MFMAs are written out as instructions: at one wave per
// SIMD the compiler would keep every accumulator in AGPRs and copy), O accumulates in AGPRs.
//
// Softmax: statistics and accumulators are fp32, probabilities are rounded to bf16 for the second MFMA.  The exponent
// reference m of a query is fixed before the key loop, on its first 32 scores: any reference gives the same quotient
// O / l, a stale one merely lets probabilities exceed 1.  Each step only notes whether a block of probabilities summed
// to more than 16 * 2^FA_SLACK; a workgroup in which that happened runs once more with the exact row maxima as
// references.  On the usual path a lane never needs the other lane half and O is never rescaled.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace vl {

constexpr int FA_BK = 64;         // keys per tile (two blocks of 32)
constexpr int FA_QW = 64;         // queries per wave
constexpr int FA_THREADS = 256;
constexpr int FA_SLOTS = 4;
constexpr float FA_SLACK = 8.0f;  // how far (base 2) scores may outgrow the exponent reference before the workgroup repeats

#define FA_LDS(p) ((__attribute__((address_space(3))) void*)(p))
constexpr int FA_WAIT_VM = 0x0F70;      // s_waitcnt vmcnt(0), other counters untouched (gfx9 encoding)

int attn_mfma_heads_per_wg(int hq, int hkv) {
    const int g = hq / hkv;
    return g % 4 == 0 ? 4 : (g % 2 == 0 ? 2 : 1);
}
int attn_mfma_q_span(int hq, int hkv) { return FA_QW * 4 / attn_mfma_heads_per_wg(hq, hkv); }

template <int HD, int HPW>
__global__ __launch_bounds__(FA_THREADS, 1) void attn_mfma_kernel(const bf16* __restrict__ qkv, int64_t n_rows,
                                                               const bf16* __restrict__ vt, int64_t ldv,
                                                               const AttnTile* __restrict__ tiles,
                                                               bf16* __restrict__ out, int hq, int hkv, float scale_log2e,
                                                               bool out_tiled) {
#if defined(__HIP_DEVICE_COMPILE__)     // the host pass needs the launch stub only; the body uses device-only types
    constexpr int KSTEPS = HD / 16;               // MFMA k-steps over the head dimension
    constexpr int DB = HD / 32;                   // 32-channel output blocks
    constexpr int KROW = HD * 2;                  // bytes per key row in LDS
    constexpr int KCPR = HD / 8;                  // 16-byte chunks per key row (16 or 8)
    constexpr int K_BYTES = FA_BK * KROW;         // K tile
    constexpr int V_BYTES = HD * FA_BK * 2;       // V^T tile: HD rows of 64 keys (128 bytes)
    constexpr int SLOT = K_BYTES + V_BYTES;
    constexpr int K_RPI = 1024 / KROW;            // key rows filled by one 1 KB load instruction
    constexpr int NI_K = FA_BK / K_RPI / 4;       // load instructions per wave and tile, K
    constexpr int NI_V = HD / 8 / 4;              //                                      V^T (8 rows per instruction)
    __shared__ __align__(1024) unsigned char ring[FA_SLOTS * SLOT];

    // Workgroup ids are dealt round-robin to the 8 XCDs.  id = tile * n_groups + x with x -> (KV head x % hkv, head
    // group x / hkv inside it): when hkv is a multiple of 8 every XCD keeps meeting the same KV heads, whose keys and
    // values then stay in that XCD's L2 while the query tiles (longest first) walk over them.
    const int n_groups = hq / HPW;
    const int gx = blockIdx.x % n_groups;
    const AttnTile t = tiles[blockIdx.x / n_groups];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, half = lane >> 5;
    const int g = gx % hkv;                       // KV head
    const int head = g * (hq / hkv) + (gx / hkv) * HPW + wave % HPW;
    const int qs = wave / HPW;                    // 64-query sub-tile of this wave
    const int64_t pitch = (int64_t)(hq + 2 * hkv) * HD;

    // ---- this lane's two queries (clamped into the tile; rows past q_rows are computed and dropped)
    int q_pos[2];
    bf16x8 qf[2][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int q_idx = min(qs * FA_QW + qb * 32 + lq, t.q_rows - 1);
        q_pos[qb] = t.pos0 + q_idx;
        const bf16* qp = qkv + (int64_t)(t.q_row0 + q_idx) * pitch + (int64_t)head * HD + half * 8;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) qf[qb][s] = *(const bf16x8*)(qp + s * 16);
    }
    const int wave_first_pos = t.pos0 + qs * FA_QW;

    // ---- tile loads: lane -> (row, physical chunk) of the 1 KB piece its wave fills; the global side applies the swizzle.
    // Buffer loads (base in scalar registers, 32-bit lane offsets) straight into LDS.
    const int n_tiles = (t.kv_len + FA_BK - 1) / FA_BK;
    const bf16* kseq = qkv + (int64_t)t.kv_row0 * pitch + (int64_t)hq * HD + (int64_t)g * HD;
    const bf16* vseq = vt + (int64_t)g * HD * ldv + t.vt_col0;
    // bytes from those two addresses to the end of their buffers (saturated; a sequence spans less than 4 GB, which
    // the launcher checks): a descriptor that starts at a tile and ends with the buffer makes rows past the end read
    // as zeros (they are masked anyway) instead of needing a clamp per lane
    const uint32_t k_total = (uint32_t)min(((int64_t)(n_rows - t.kv_row0) * pitch - (int64_t)(hq + g) * HD) * 2, (int64_t)0xFFFFFFFFll);
    const uint32_t v_total = (uint32_t)min(((int64_t)HD * ldv - t.vt_col0) * 2, (int64_t)0xFFFFFFFFll);
    const uint32_t row_bytes = (uint32_t)pitch * 2;
    const int k_row = wave * K_RPI + lane / KCPR;                     // + 4 * K_RPI * i
    const int k_swz = KCPR == 16 ? (k_row & 15) : ((k_row >> 1) & 7);
    const int v_row = wave * 8 + (lane >> 3);                         // + 32 * i
    uint32_t k_lane[NI_K], v_lane[NI_V];                              // byte offsets from the tile's first key, per lane
#pragma unroll
    for (int i = 0; i < NI_K; ++i) k_lane[i] = (uint32_t)(k_row + 4 * K_RPI * i) * row_bytes + ((lane % KCPR) ^ k_swz) * 16;
#pragma unroll
    for (int i = 0; i < NI_V; ++i) v_lane[i] = (uint32_t)(v_row + 32 * i) * (uint32_t)ldv * 2 + ((lane & 7) ^ ((v_row >> 1) & 7)) * 16;
    // One tile = NI_K + NI_V load instructions per wave (buffer loads that write LDS directly: 64 lanes x 16 bytes land at
    // M0 + 16 * lane).  They are written out by hand: the compiler would order every later LDS read behind a full wait
    // for a load of this kind that it knows of, which defeats spreading the loads over the slots of a step (issued back
    // to back they hold the wave for some 400 cycles per tile).  Completion is awaited explicitly: s_waitcnt vmcnt(0)
    // before the barrier that publishes a tile.  The descriptors are scalar; a tile that does not exist gets empty
    // ones, so its loads touch no memory (they fill a free slot with zeros) and the code needs no branch.
    constexpr int NPIECE = NI_K + NI_V;
    auto tile_descriptors = [&](int tile, u32x4& k_rsrc, u32x4& v_rsrc) {
        const uint32_t k_skip = (uint32_t)tile * FA_BK * row_bytes, v_skip = (uint32_t)tile * FA_BK * 2;
        const bool there = tile < n_tiles;
        const uint32_t k_left = (there && k_total > k_skip) ? k_total - k_skip : 0u, v_left = (there && v_total > v_skip) ? v_total - v_skip : 0u;
        const uint64_t ka = (uint64_t)kseq + k_skip, va = (uint64_t)vseq + v_skip;
        // raw buffer descriptor: base, stride 0, bytes, data format
        auto uni = [](uint32_t x) -> uint32_t { return (uint32_t)__builtin_amdgcn_readfirstlane(x); };
        k_rsrc = u32x4{uni((uint32_t)ka), uni((uint32_t)(ka >> 32) & 0xffffu), uni(k_left), 0x00020000u};
        v_rsrc = u32x4{uni((uint32_t)va), uni((uint32_t)(va >> 32) & 0xffffu), uni(v_left), 0x00020000u};
    };
    const uint32_t ring_lds = (uint32_t)(uintptr_t)FA_LDS(ring) + wave * 1024;
    auto issue_piece = [&](int tile, int piece, const u32x4& k_rsrc, const u32x4& v_rsrc) {
        const uint32_t dst = ring_lds + (tile & (FA_SLOTS - 1)) * SLOT + (piece < NI_K ? piece * 4096 : K_BYTES + (piece - NI_K) * 4096);
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
                     :: "v"(piece < NI_K ? k_lane[piece] : v_lane[piece - NI_K]), "s"(piece < NI_K ? k_rsrc : v_rsrc), "s"(dst)
                     : "m0");                                 // the statement sets M0: the compiler must not keep a value there
    };
    auto issue_tile = [&](int tile) {
        u32x4 k_rsrc, v_rsrc;
        tile_descriptors(tile, k_rsrc, v_rsrc);
#pragma unroll
        for (int i = 0; i < NPIECE; ++i) issue_piece(tile, i, k_rsrc, v_rsrc);
    };

    // ---- fragment read offsets inside a slot
    const int prow = (lq & ~12) | ((lq & 4) << 1) | ((lq & 8) >> 1);  // key row this lane feeds to the first MFMA
    const int kx = half ^ (KCPR == 16 ? (prow & 15) : ((prow >> 1) & 7));
    int k_off[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) k_off[s] = prow * KROW + (((2 * s) ^ kx) << 4);      // + 32 * KROW * kb
    const int vx = half ^ ((lq >> 1) & 7);
    int v_off[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) v_off[kb][s2] = K_BYTES + lq * 128 + (((4 * kb + 2 * s2) ^ vx) << 4);   // + 4096 * b

    f32x16 o[DB][2];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[b][qb][r] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};                   // this lane half's share of the row sums

    // One pipeline step = NSLOT matrix instructions, each followed by its share of the vector work of the step and
    // fenced for the scheduler, so the instruction stream alternates between the two pipes exactly as written:
    //   slots 0 .. NS-1      S_next[qb] (+)= K fragment s x Q[qb][s]                     s = slot / 2, qb = slot % 2
    //   slots NS .. NSLOT-1  O[b][qb]    += V^T fragment (s2, b) x P_prev[qb][s2]        i = slot - NS: s2 = i / (2 DB), b = (i / 2) % DB, qb = i % 2
    //   fragment i (K fragments first, then V^T fragments) feeds slots 2 i and 2 i + 1 and is read FA_AHEAD fragments
    //   early into a ring of eight registers quads; the last reads of a step are the first K fragments of the NEXT
    //   step (block 1 - KB of the tile in `nkslot`), so no step starts by waiting for LDS
    //   every_slot(slot): the caller's share of other work (the first step of a tile spreads the loads of the tile after
    //   next over its slots)
    //   vector work: slot e turns score(s) e of S_cur into probabilities; every second score closes a pair (rounding
    //   to bf16, row sum of the rounded values)
    constexpr int NS = 2 * KSTEPS, NSLOT = NS + 4 * DB, NFRAG = NSLOT / 2;
    constexpr int FA_AHEAD = HD == 128 ? 5 : 4;      // <= KSTEPS: the early reads for the next step are all K fragments
    constexpr int EPS = 32 / NSLOT;                // scores per slot (1 or 2)
    bf16x8 fr[8];
    auto step = [&](const unsigned char* kslot, const unsigned char* vslot, const unsigned char* nkslot, auto kb_c,
                    const f32x16 (&Sc)[2], f32x16 (&Sn)[2], const u32x4 (&Pp)[2][2], u32x4 (&Pc)[2][2], auto&& every_slot) {
        constexpr int KB = decltype(kb_c)::value;
        auto read_frag = [&](int i) {
            if (i < KSTEPS) fr[i & 7] = *(const bf16x8*)(kslot + KB * 32 * KROW + k_off[i]);
            else if (i < NFRAG) { const int j = i - KSTEPS; fr[i & 7] = *(const bf16x8*)(vslot + v_off[KB][j / DB] + (j % DB) * 4096); }
            else fr[i & 7] = *(const bf16x8*)(nkslot + (1 - KB) * 32 * KROW + k_off[i - NFRAG]);
        };
        float pe[4] = {0.f, 0.f, 0.f, 0.f};
        // closes pair u of S_cur: adds its two probabilities to the row sum and rounds them to bf16.  (Plain adds: the
        // packed dot-product instructions share the matrix pipe and would not run beside the MFMAs.)
        auto close_pair = [&](int u) {
            const int eq = u >> 3, r0 = 2 * (u & 7);
            const f32x2 pp = {pe[(2 * u) & 3], pe[(2 * u + 1) & 3]};
            l_run[eq] += pp[0];
            l_run[eq] += pp[1];
            uint32_t wi = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, bf16x2));
            asm volatile("" : "+v"(l_run[eq]), "+v"(wi));             // pinned to this slot: nothing may sink below
            Pc[eq][r0 >> 3][(r0 & 7) >> 1] = wi;
        };
#pragma unroll
        for (int slot = 0; slot < NSLOT; ++slot) {
            const int i = slot >> 1, qb = slot & 1;
            if (qb == 0) read_frag(i + FA_AHEAD);
            every_slot(slot);
            // ---- matrix pipe
            if (slot < NS) {
                if (i == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(Sn[qb]) : "v"(fr[i & 7]), "a"(qf[qb][i]));
                else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(Sn[qb]) : "v"(fr[i & 7]), "a"(qf[qb][i]));
            } else {
                const int j = i - KSTEPS, s2 = j / DB, b = j % DB;
                o[b][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i & 7], __builtin_bit_cast(bf16x8, Pp[qb][s2]), o[b][qb], 0, 0, 0);
            }
            // ---- vector pipe: exponentials of this slot's score(s); the pair finished one slot ago is closed (its
            // exponentials have left the transcendental unit by now)
#pragma unroll
            for (int k = 0; k < EPS; ++k) {
                const int e = slot * EPS + k, eq = e >> 4, r = e & 15;
                if ((e & 1) == 0 && e >= 2) close_pair(e / 2 - 1);
                pe[e & 3] = __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[eq][r], scale_log2e, -m_run[eq]));
                asm volatile("" : "+v"(pe[e & 3]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        close_pair(15);
    };
    // S^T of one block outside the pipeline (the first block; the rare second pass over the scores).  The same hand-issued
    // instruction as in `step`, so that every use of Q asks for the accumulator registers and Q stays there for the
    // whole kernel.  The compiler does not know these are matrix instructions and inserts none of the wait states the
    // hardware needs after a vector write of an operand (it may copy Q into place right before a use: here it does,
    // when registers are short) or before a vector read of the result.  Not time-critical, so each instruction waits
    // first and the last one is left to drain; `step` has no such padding, and the generated code is checked at build
    // time for operands written next to its instructions.
    auto block_scores = [&](const unsigned char* slot, int kb, f32x16 (&S)[2]) {
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const bf16x8 kf = *(const bf16x8*)(slot + kb * 32 * KROW + k_off[s]);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (s == 0) asm volatile("s_nop 3\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(S[qb]) : "v"(kf), "a"(qf[qb][s]));
                else asm volatile("s_nop 3\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(S[qb]) : "v"(kf), "a"(qf[qb][s]));
            }
        }
        asm volatile("s_nop 15\n\ts_nop 7" : "+v"(S[0]), "+v"(S[1]));
    };
    // causal mask of a block that reaches past the wave's first query
    auto mask_block = [&](f32x16 (&S)[2], int key0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int d = q_pos[qb] - key0 - 8 * half;                // key of register r = key0 + 8*half + 16*(r/8) + r%8
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (16 * (r >> 3) + (r & 7) > d) S[qb][r] = -INFINITY;
        }
    };
    // this lane's maxima of a block's raw scores, folded into mx
    auto block_max = [&](const f32x16 (&S)[2], float (&mx)[2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx[qb] = fmaxf(mx[qb], S[qb][r]);
    };
    auto fenced_barrier = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // The exponent reference of a query is fixed before the key loop: the maximum of its first 32 scores.  Later
    // scores may exceed it; the probabilities then exceed 1, which is harmless until they overflow.  Each step only
    // notes whether a lane's block of 16 probabilities summed to more than 16 * 2^FA_SLACK (or to something that is not
    // a number).  If any wave of the workgroup noted that, the workgroup runs again with the exact row maxima as
    // references, found by one extra pass over the scores; then no probability exceeds 1.
    __shared__ int vote;
    if (tid == 0) vote = 0;
    bool noted = false;
    for (int attempt = 0; attempt < 2; ++attempt) {
        float mx[2] = {-INFINITY, -INFINITY};
        f32x16 Sa[2], Sb[2];
        if (attempt == 1) {
            // second pass: exact row maxima over all keys
            for (int t2 = 0; t2 < n_tiles; ++t2) {
                const unsigned char* cur = ring + (t2 & (FA_SLOTS - 1)) * SLOT;
                issue_tile(t2);
                __builtin_amdgcn_s_waitcnt(FA_WAIT_VM);
                fenced_barrier();
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    block_scores(cur, kb, Sa);
                    if (t2 * FA_BK + 32 * kb + 31 > wave_first_pos) mask_block(Sa, t2 * FA_BK + 32 * kb);
                    block_max(Sa, mx);
                }
            }
            fenced_barrier();                      // every wave is done with the ring before it is refilled
        }

        // ---- tiles 0 and 1 requested, S of block 0
        issue_tile(0);
        if (n_tiles > 1) issue_tile(1);
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[b][qb][r] = 0.f;
        u32x4 Pa[2][2], Pb[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) Pb[qb][s2] = u32x4{0u, 0u, 0u, 0u};
        __builtin_amdgcn_s_waitcnt(FA_WAIT_VM);    // everything requested so far has landed (whatever order it was issued in)
        fenced_barrier();
        block_scores(ring, 0, Sa);
        mask_block(Sa, 0);                         // block 0 always meets the diagonal or lies below it: cheap either way
        if (attempt == 0) block_max(Sa, mx);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {           // key 0 is visible to every query: the maxima are finite
            m_run[qb] = fmaxf(mx[qb], __shfl_xor(mx[qb], 32, WAVE)) * scale_log2e;
            l_run[qb] = 0.f;
        }
        // the first fragments of the first pipeline step (second block of tile 0)
        // (issued in this order and as the last LDS reads before the loop, exactly as every step leaves them)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < FA_AHEAD; ++i) {
            fr[i] = *(const bf16x8*)(ring + 32 * KROW + k_off[i]);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- tile t2: blocks 2 t2 (kb 0, scores in Sa) and 2 t2 + 1 (kb 1, scores in Sb)
        constexpr float bound = 16.0f * (float)(1 << (int)FA_SLACK);
        for (int t2 = 0; t2 < n_tiles; ++t2) {
            const unsigned char* cur = ring + (t2 & (FA_SLOTS - 1)) * SLOT;
            const unsigned char* prev = ring + ((t2 > 0 ? t2 - 1 : 0) & (FA_SLOTS - 1)) * SLOT;
            const int t_next = min(t2 + 1, n_tiles - 1);
            const unsigned char* next = ring + (t_next & (FA_SLOTS - 1)) * SLOT;
            // tile t2+1 (requested one tile ago) has landed; every wave has left tile t2-2, whose slot takes tile t2+2
            __builtin_amdgcn_s_waitcnt(FA_WAIT_VM);
            fenced_barrier();
            u32x4 k_rsrc, v_rsrc;
            tile_descriptors(t2 + 2, k_rsrc, v_rsrc);

            // block 2 t2: the matrix pipe computes S of this tile's second block and O += V P of the previous tile's
            // second block (t2 = 0: P = 0 against the finite values of tile 0)
            const float la0 = l_run[0], la1 = l_run[1];
            constexpr int every = NSLOT / NPIECE;   // one load instruction every `every` slots
            step(cur, prev, next, std::integral_constant<int, 1>{}, Sa, Sb, Pb, Pa, [&](int slot) {
                if (slot % every == every / 2) issue_piece(t2 + 2, slot / every, k_rsrc, v_rsrc);
            });
            noted |= !(l_run[0] - la0 <= bound) | !(l_run[1] - la1 <= bound);       // (also true for a sum that is no number)
            if (t2 * FA_BK + 63 > wave_first_pos) mask_block(Sb, t2 * FA_BK + 32);

            // block 2 t2 + 1: S of the next tile's first block (the last tile recomputes its own; unused) and O += V P of kb 0
            const float lb0 = l_run[0], lb1 = l_run[1];
            step(next, cur, next, std::integral_constant<int, 0>{}, Sb, Sa, Pa, Pb, [](int) {});
            noted |= !(l_run[0] - lb0 <= bound) | !(l_run[1] - lb1 <= bound);
            if (t_next * FA_BK + 31 > wave_first_pos) mask_block(Sa, t_next * FA_BK);
        }
        // O += V P of the last block
        {
            const unsigned char* last = ring + ((n_tiles - 1) & (FA_SLOTS - 1)) * SLOT;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    const bf16x8 vf = *(const bf16x8*)(last + v_off[1][s2] + b * 4096);
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        o[b][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, Pb[qb][s2]), o[b][qb], 0, 0, 0);
                }
        }
        if (attempt == 1) break;
        // has any wave of the workgroup noted an outgrown reference?  (uniform for the workgroup: all waves repeat together)
        if (__builtin_amdgcn_ballot_w64(noted) != 0 && lane == 0) vote = 1;
        fenced_barrier();                          // also: every wave is past its last fragment read
        if (__builtin_amdgcn_readfirstlane(*(volatile int*)&vote) == 0) break;
    }

    // ---- normalise, transpose through LDS (the ring is free once every wave is past its last fragment read) and store
    // whole 16-byte pieces: lane holds query qb*32 + lq of its sub-tile, channels b*32 + 8*(r/4) + 4*half + r%4
    constexpr int OP = HD * 2 + 8;                 // row pitch of the staging rows: 8-byte writes of 32 lanes hit 64 banks
    __builtin_amdgcn_s_waitcnt(FA_WAIT_VM);        // (the zero fills of tiles past the end have landed too)
    fenced_barrier();
    unsigned char* stage = ring + wave * (FA_QW * OP);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float inv = 1.0f / (l_run[qb] + __shfl_xor(l_run[qb], 32, WAVE));
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[b][qb][rg * 4 + e] * inv);
                *(bf16x4*)(stage + (qb * 32 + lq) * OP + (b * 32 + rg * 8 + half * 4) * 2) = v;
            }
    }
    // (a wave reads back only what it wrote itself: no barrier)
    const int q_valid = t.q_rows - qs * FA_QW;     // rows of this wave's sub-tile that exist
    const int64_t orow0 = t.q_row0 + qs * FA_QW;
    if (out_tiled) {
        // tiled image: for one k-tile of 32 channels, consecutive rows are 64 bytes apart -> 16 rows = 1 KB per instruction
#pragma unroll
        for (int kt = 0; kt < HD / 32; ++kt)
#pragma unroll
            for (int i = 0; i < FA_QW / 16; ++i) {
                const int q = 16 * i + (lane >> 2), c = kt * 32 + (lane & 3) * 8;
                const bf16x4 lo = *(const bf16x4*)(stage + q * OP + c * 2), hi = *(const bf16x4*)(stage + q * OP + c * 2 + 8);
                if (q < q_valid) {
                    bf16* dst = out + tiled_off(orow0 + q, head * HD + c, (int64_t)hq * HD);
                    *(bf16x4*)dst = lo;
                    *(bf16x4*)(dst + 4) = hi;
                }
            }
    } else {
        // row-major: a row of this head is HD * 2 contiguous bytes
        constexpr int LPR = HD / 8;                // lanes per row
#pragma unroll
        for (int i = 0; i < FA_QW / (64 / LPR); ++i) {
            const int q = (64 / LPR) * i + lane / LPR, c = (lane % LPR) * 8;
            const bf16x4 lo = *(const bf16x4*)(stage + q * OP + c * 2), hi = *(const bf16x4*)(stage + q * OP + c * 2 + 8);
            if (q < q_valid) {
                bf16* dst = out + (orow0 + q) * hq * HD + head * HD + c;
                *(bf16x4*)dst = lo;
                *(bf16x4*)(dst + 4) = hi;
            }
        }
    }
#endif
}

template <int HD>
static void launch_hd(const bf16* qkv, int64_t n_rows, const bf16* vt, int64_t ldv, const AttnTile* tiles, int n_tiles, bf16* out,
                      int hq, int hkv, float scale_log2e, bool out_tiled, hipStream_t s) {
    const int hpw = attn_mfma_heads_per_wg(hq, hkv);
    const unsigned grid = (unsigned)n_tiles * (unsigned)(hq / hpw);
    if (hpw == 4) attn_mfma_kernel<HD, 4><<<grid, FA_THREADS, 0, s>>>(qkv, n_rows, vt, ldv, tiles, out, hq, hkv, scale_log2e, out_tiled);
    else if (hpw == 2) attn_mfma_kernel<HD, 2><<<grid, FA_THREADS, 0, s>>>(qkv, n_rows, vt, ldv, tiles, out, hq, hkv, scale_log2e, out_tiled);
    else attn_mfma_kernel<HD, 1><<<grid, FA_THREADS, 0, s>>>(qkv, n_rows, vt, ldv, tiles, out, hq, hkv, scale_log2e, out_tiled);
}

bool attn_mfma_fits(int hq, int hkv, int hd, int64_t max_seq_len) {
    return max_seq_len * (int64_t)(hq + 2 * hkv) * hd * 2 < (int64_t)0xFFFFFFFFll;
}

void launch_attn_mfma(const void* qkv, int64_t n_rows, const void* vt, int64_t ldv, const AttnTile* tiles, int n_tiles,
                      void* out, int hq, int hkv, int hd, hipStream_t s, bool out_tiled) {
    if (n_tiles <= 0) return;
    const float scale_log2e = (1.0f / sqrtf((float)hd)) * 1.4426950408889634f;
    if (hd == 128) launch_hd<128>((const bf16*)qkv, n_rows, (const bf16*)vt, ldv, tiles, n_tiles, (bf16*)out, hq, hkv, scale_log2e, out_tiled, s);
    else launch_hd<64>((const bf16*)qkv, n_rows, (const bf16*)vt, ldv, tiles, n_tiles, (bf16*)out, hq, hkv, scale_log2e, out_tiled, s);
}

}  // namespace vl
