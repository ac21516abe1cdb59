// Host-side launchers of the gfx950 kernels.  Every pointer is a device pointer unless it says otherwise;
// every launcher enqueues on `s` and returns without synchronising.  Shapes are validated by the caller
// (engine.hip) before any launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/verillm.h"

namespace vl {

// ---- elementwise / row kernels (kernels_rows.hip) ------------------------------------------------
// resid[n,:] = E[id, :] with id = tok[row_tok ? row_tok[n] : n].  An id outside [0,vocab) reads row 0 instead and
// clears valid[dst ? dst[n] : n] (valid may be NULL); activations therefore stay finite whatever the ids are.
void launch_embed(const void* E, int dtype, const int32_t* tok, const int32_t* row_tok, float* resid,
                  uint8_t* valid, const int32_t* dst, int64_t rows, int d, int vocab, hipStream_t s);
// out[n,:] = x[n,:] * rsqrt(mean(x[n,:]^2) + eps) * gain, written in `dtype`; out_tiled: `out` is the tiled image
// of [rows][d] (see tiled_off) instead of row-major.
void launch_rmsnorm(const float* x, const float* gain, void* out, int dtype, int64_t rows, int d, float eps,
                    hipStream_t s, bool out_tiled = false);
// dst (tiled image of a [.][K] bf16 matrix) <- rows [0, rows) of src (row-major [rows][K]); source row r lands on row
// row0 + r, or, with interleave > 0, on row 2*ib*(r/ib) + (interleave == 2 ? ib : 0) + r%ib with ib = 32 (the gate /
// up interleaving), in both cases counted from row0.
void launch_retile(const void* src, void* dst, int64_t rows, int K, int64_t row0, int interleave, hipStream_t s);
// Rotate query and key heads of qkv [rows][(hq+2hkv)*hd] in place using the cos/sin table
// cs[pos][hd/2] (float2 = cos, sin).  With cache_row != NULL the rotated keys and the values of row n are also
// copied to row cache_row[n] of kcache / vcache ([cache rows][hkv*hd], same dtype).
void launch_rope(void* qkv, int dtype, const int32_t* pos, const float2* cs, int64_t rows, int hq, int hkv,
                 int hd, hipStream_t s, void* kcache = nullptr, void* vcache = nullptr, const int32_t* cache_row = nullptr);
// vt[g][c][ vt_col[n] ] = V head g, channel c of token n (bf16); ldv = row pitch of vt in elements.
void launch_transpose_v(const void* qkv, void* vt, const int32_t* vt_col, int64_t rows, int hq, int hkv, int hd,
                        int64_t ldv, hipStream_t s);
// resid[n, :] = in[n, :] upcast exactly from `dtype` (the recorded states a segment starts from).
void launch_load_hidden(const void* in, int dtype, float* resid, int64_t rows, int d, hipStream_t s);
// out[(dst ? dst[n] : n), :] = resid[n, :] converted to `dtype`.
void launch_store_hidden(const float* resid, void* out, int dtype, const int32_t* dst, int64_t rows, int d,
                         hipStream_t s);
// Token-by-token path: copy rows [*off, *off + rows) of four index arrays into cur[k * stride + i], then *off += rows.
void launch_step_prologue(const int32_t* a0, const int32_t* a1, const int32_t* a2, const int32_t* a3, int32_t* cur, int32_t* off,
                          int rows, int stride, hipStream_t s);
void launch_scatter_i32(const int32_t* src, int32_t* out, const int32_t* dst, int64_t rows, hipStream_t s);
void launch_fill_u8(uint8_t* p, uint8_t v, int64_t n, hipStream_t s);

// ---- simple tiled GEMM on the vector ALUs (kernels_gemm_simple.hip) ------------------------------
enum EpiKind { EPI_STORE = 0, EPI_STORE_F32 = 1, EPI_ADD_RESID = 2, EPI_SWIGLU = 3, EPI_QKV_ROPE = 4, EPI_ARGMAX = 5 };
// C[M,N] = A[M,K] * W[N,K]^T, fp32 accumulate.  A and W are `dtype`.
//   EPI_STORE     : out [M][N] in dtype
//   EPI_STORE_F32 : out [M][N] float
//   EPI_ADD_RESID : out [M][N] float, out += C
//   EPI_SWIGLU    : W rows interleave gate/up in blocks of `ib` rows (ib gate rows, ib up rows, ...);
//                   out [M][N/2] in dtype = silu(gate) * up
void launch_gemm_simple(const void* A, const void* W, int dtype, int M, int N, int K, int epi, void* out, int ib,
                        hipStream_t s);

// ---- bf16 matrix-core GEMM (kernels_gemm_mfma.hip) -----------------------------------------------
// Same contract as launch_gemm_simple with dtype = bf16; K % 64 == 0; EPI_SWIGLU interleaves in blocks of 32
// rows and needs N % 64 == 0.
// layout: bit 0 = A is a tiled image, bit 1 = W is, bit 2 = the SwiGLU output is written as one (see tiled_off).
enum GemmLayout { GL_A_TILED = 1, GL_W_TILED = 2, GL_OUT_TILED = 4 };
void launch_gemm_mfma(const void* A, const void* W, int M, int N, int K, int epi, void* out, hipStream_t s, int layout = 0);

// LM head with the argmax in the epilogue: the logits never reach memory.  The GEMM runs transposed (rows = vocabulary,
// columns = tokens), so that a lane's accumulators are 64 vocabulary entries of ONE token and the maximum over them needs
// no cross-lane work; every wave reduces its 128 x 64 block to one (maximum, lowest index attaining it) per token.
//   pmax, pidx : [parts][ld], parts = ceil(vocab / 128); part p covers vocabulary rows 128 p .. 128 p + 127
//   tok, ztok  : tok[n] (may be NULL) is a vocabulary index per token whose logit is also wanted: ztok[n] receives it
//                (entries with tok[n] outside [0, vocab) are left untouched)
struct ArgmaxParts {
    float* pmax;
    int32_t* pidx;
    const int32_t* tok;
    float* ztok;
    int64_t ld;
};
inline int argmax_parts(int vocab) { return (vocab + 127) / 128; }
// Wlm [vocab][K] and X [tokens][K] as for launch_gemm_mfma's W and A (layout bits GL_W_TILED / GL_A_TILED)
void launch_gemm_mfma_argmax(const void* X, const void* Wlm, int tokens, int vocab, int K, const ArgmaxParts& parts, hipStream_t s,
                             int layout = 0);

// ---- bf16 weight-streaming GEMM for M <= 64 rows (kernels_gemm_skinny.hip) --------------------------
// Same contract; K % 32 == 0; EPI_SWIGLU needs N % 64 == 0.
constexpr int GEMM_SKINNY_MAX_M = 64;
void launch_gemm_skinny(const void* A, const void* W, int M, int N, int K, int epi, void* out, hipStream_t s, int layout = 0);
// The q/k/v projection of a decode step with the rotary embedding and the KV-cache append in its epilogue:
// W = [Wq; Wk; Wv] ((hq + 2 hkv) * hd rows), qkv [M][(hq + 2 hkv) * hd] receives rotated q and k and plain v; row m's
// rotated key and its value also go to row cache_row[m] of kcache / vcache ([cache rows][hkv * hd]).  pos, cache_row:
// device, [M]; cs: cos/sin table [position][hd / 2].  Needs hd % 32 == 0 and M <= GEMM_SKINNY_MAX_M.
// With norm_gain != NULL, A is instead the fp32 residual [M][K] (row-major) and the kernel applies RMSNorm(gain, eps)
// to it first (allowed when gemm_skinny_norm_supported(M, K)).
bool gemm_skinny_qkv_rope_supported(int M, int hd);
void launch_gemm_skinny_qkv_rope(const void* A, const void* W, int M, int K, void* qkv, const int32_t* pos, const float2* cs,
                                 const int32_t* cache_row, void* kcache, void* vcache, int hq, int hkv, int hd, hipStream_t s,
                                 int layout = 0, const float* norm_gain = nullptr, float eps = 0.f);
bool gemm_skinny_norm_supported(int M, int K);

// ---- attention ------------------------------------------------------------------------------------
// One wave per (query row, query head), online softmax over keys 0..npos[row].
//   q    : [rows][q_stride] elements, head j at offset j*hd
//   k, v : key/value t of row r, kv head g at  base[(kv_row0[r] + t) * kv_stride + g*hd]
void launch_attn_rowwise(const void* q, int64_t q_stride, const void* k, const void* v, int64_t kv_stride,
                         const int32_t* kv_row0, const int32_t* npos, void* out, int dtype, int64_t rows, int hq,
                         int hkv, int hd, hipStream_t s, bool out_tiled = false);

// bf16, one workgroup per (query row, KV head), all query heads of the group together (kernels_attn_decode.hip).
// Same addressing as launch_attn_rowwise; needs head_dim 64 or 128 and Hq / Hkv in {1, 2, 4, 8}.
bool attn_decode_supported(int hq, int hkv, int hd);
void launch_attn_decode(const void* q, int64_t q_stride, const void* k, const void* v, int64_t kv_stride,
                        const int32_t* kv_row0, const int32_t* npos, void* out, int64_t rows, int hq, int hkv, int hd,
                        hipStream_t s, bool out_tiled = false);
// Causal GQA flash attention on the matrix cores over packed sequences.
//   qkv bf16 [N][(hq+2hkv)*hd], vt bf16 [hkv][hd][ldv] (values transposed, column = vt column of the token),
//   tiles: host-built work list (see engine), out bf16 [N][hq*hd].
struct AttnTile { int32_t q_row0, q_rows, kv_row0, kv_len, vt_col0, pos0; };  // one query tile of a sequence:
//   q_row0  packed row of its first query, q_rows valid queries (<= attn_mfma_q_span), pos0 position of the first query
//           (a multiple of the span), kv_row0 packed row of the sequence's first token, kv_len = pos0 + q_rows keys are
//   visible to the tile, vt_col0 column of the sequence's first token in vt (a multiple of 8)
// Queries per tile for this head geometry: 64, 128 or 256 (a workgroup serves 4, 2 or 1 query heads of one KV head).
int attn_mfma_q_span(int hq, int hkv);
// The kernel addresses a sequence's keys with 32-bit byte offsets: the longest sequence it can take.
bool attn_mfma_fits(int hq, int hkv, int hd, int64_t max_seq_len);
void launch_attn_mfma(const void* qkv, int64_t n_rows, const void* vt, int64_t ldv, const AttnTile* tiles, int n_tiles,
                      void* out, int hq, int hkv, int hd, hipStream_t s, bool out_tiled = false);

// ---- compare / argmax / flags (kernels_compare.hip) ------------------------------------------------
void launch_compare(const float* h_hat, const void* committed, int hidden_dtype, int64_t rows, int d, float tol_rel,
                    float tol_abs, vl_tok_stats* stats, uint8_t* ok_and, uint8_t* ok_set, hipStream_t s,
                    const vl_bit_rule* rule = nullptr, vl_bit_stats* bit_stats = nullptr);
void launch_argmax(const float* logits, int64_t rows, int vocab, const int32_t* committed, float margin,
                   int32_t* out_argmax, float* out_gap, uint8_t* out_ok, hipStream_t s);
// The same outputs from the per-part maxima of launch_gemm_mfma_argmax (parts.tok must have been `committed`).
void launch_argmax_reduce(const ArgmaxParts& parts, int64_t rows, int vocab, const int32_t* committed, float margin,
                          int32_t* out_argmax, float* out_gap, uint8_t* out_ok, hipStream_t s);
// ---- Merkle commitment (kernels_merkle.hip) -----------------------------------------------------------
// roots[r][32] = SHA-256 Merkle root over the d canonical-float32 scalars of states row r (dtype VL_F32 / VL_BF16);
// d <= 16384.
void launch_merkle_roots(const void* states, int dtype, int64_t rows, int d, uint8_t* roots, hipStream_t s);
// ceil(log2 d): the longest inclusion proof
int merkle_depth(int d);
// Opening q discloses element sel_idx[q] of row sel_row[q]: values[q] (may be NULL) and the sibling digests, leaf level
// first, in paths[q][depth][32] (entries past the proof's length are zero).  scratch: count * 2 * d * 32 bytes.
void launch_merkle_open(const void* states, int dtype, int d, const int32_t* sel_row, const int32_t* sel_idx, int count,
                        uint32_t* scratch, uint8_t* paths, float* values, hipStream_t s);

struct DevSummary { unsigned long long n_rejected, n_hidden_reject, n_token_reject; float max_rel, max_abs, mean_mae; };
void launch_finalize(const uint8_t* hid_ok, const uint8_t* tok_ok, const vl_tok_stats* stats, int C, int64_t rows,
                     uint8_t* flags, DevSummary* out, hipStream_t s);

}  // namespace vl
