// The comparison stage (Section 5.7 "Comparison and On-Chain Commitment"): elementwise discrepancy
// Delta = S_hat - S between the recomputed and the committed hidden states, reduced per token to
// rel-L2 / max-abs / mean-abs / mean-signed and thresholded; the TokenMatch check on the logits; the final
// per-position flags and the batch summary.  All three kernels are pure HBM streaming: one wave owns one
// row (compare) or one workgroup owns one row (argmax), every load is a contiguous 16 bytes per lane, and all
// reductions are butterfly shuffles in a fixed order, so results are bit-identical from run to run.
#include "common.h"
#include "kernels.h"

namespace vl {

// ---------------------------------------------------------------- compare: one wave per token row
template <typename TC> struct Load8;
template <> struct Load8<bf16> {
    static __device__ __forceinline__ void load(const bf16* p, float (&v)[8]) {
        const bf16x8 t = *(const bf16x8*)p;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
    }
};
template <> struct Load8<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
        const float4 a = ((const float4*)p)[0], b = ((const float4*)p)[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};

// Bit-aware counts of Section 7 ("Bit-aware statistical comparison") and of the offline battery of Appendix A.1,
// taken in the same pass when BITS is set: both operands are canonical float32, split into exponent (bits 30..23)
// and mantissa (bits 22..0) fields; per row
//   exact          identical bit patterns
//   exp_mismatch   exponent fields differ                                      (P_e  = exp_mismatch / d)
//   mismatch_close among those, |Delta| <= e_w                                 (P_m  = mismatch_close / exp_mismatch)
//   match_small    among equal exponents, mantissa fields <= mant_tol apart    (P_w  = match_small / (d - exp_mismatch))
//   small / large  |Delta| <= q_small, |Delta| > tau_large                     (Q_small, Z_large)
// and the acceptance rule P_e < pe_max, P_m > pm_min, P_w > pw_min, |mean Delta| <= eps_max, Q_small >= q_small_min,
// Z_large <= z_large_max, each ratio test taken as count vs bound * size in fp32; a ratio over an empty set passes.
struct BitParams {
    float e_w, q_small, tau_large;
    int mant_tol;                                  // e_m << step_log2, clamped to the largest mantissa distance
    float pe_max, pm_min, pw_min, eps_max, q_small_min, z_large_max;
};

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

template <typename TC, bool BITS>
__global__ __launch_bounds__(256) void compare_kernel(const float* __restrict__ h_hat, const TC* __restrict__ h_star,
                                                      int64_t rows, int d, float tol_rel, float tol_abs,
                                                      vl_tok_stats* __restrict__ stats, uint8_t* __restrict__ ok_and,
                                                      uint8_t* __restrict__ ok_set, BitParams bp,
                                                      vl_bit_stats* __restrict__ bit_stats) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;                      // whole wave leaves together; no barrier below
    const float* a = h_hat + row * (int64_t)d;
    const TC* b = h_star + row * (int64_t)d;
    float e2 = 0.f, n2 = 0.f, e1 = 0.f, es = 0.f, emax = 0.f;
    int c_exact = 0, c_mis = 0, c_close = 0, c_msmall = 0, c_small = 0, c_large = 0;
    const int chunks = d >> 3;
#pragma unroll 4
    for (int c = lane; c < chunks; c += WAVE) {
        float x[8], y[8];
        Load8<float>::load(a + 8 * c, x);
        Load8<TC>::load(b + 8 * c, y);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float dl = x[i] - y[i];
            e2 = fmaf(dl, dl, e2);
            n2 = fmaf(x[i], x[i], n2);
            e1 += fabsf(dl);
            es += dl;
            emax = fmaxf(emax, fabsf(dl));        // fmaxf drops NaN; a NaN row is recovered from e2 below
            if (BITS) {
                const uint32_t ux = __float_as_uint(x[i]), uy = __float_as_uint(y[i]);
                const bool mis = ((ux ^ uy) & 0x7F800000u) != 0;
                const int md = abs((int)(ux & 0x7FFFFFu) - (int)(uy & 0x7FFFFFu));
                const float ad = fabsf(dl);
                c_exact += (ux == uy);
                c_mis += mis;
                c_close += mis && (ad <= bp.e_w);
                c_msmall += !mis && (md <= bp.mant_tol);
                c_small += (ad <= bp.q_small);
                c_large += (ad > bp.tau_large);
            }
        }
    }
    e2 = wave_sum(e2);
    n2 = wave_sum(n2);
    e1 = wave_sum(e1);
    es = wave_sum(es);
    emax = wave_max(emax);
    if (BITS) {
        c_exact = wave_sum_i(c_exact);
        c_mis = wave_sum_i(c_mis);
        c_close = wave_sum_i(c_close);
        c_msmall = wave_sum_i(c_msmall);
        c_small = wave_sum_i(c_small);
        c_large = wave_sum_i(c_large);
    }
    if (lane == 0) {
        const float rel = sqrtf(e2) / fmaxf(sqrtf(n2), 1e-30f);
        if (e2 != e2) emax = e2;                  // NaN anywhere in the row -> max_abs is NaN
        const float inv_d = 1.0f / (float)d;
        vl_tok_stats st;
        st.rel_l2 = rel;
        st.max_abs = emax;
        st.mean_abs = e1 * inv_d;
        st.mean_signed = es * inv_d;
        if (stats) stats[row] = st;
        uint8_t ok = (rel <= tol_rel) && (emax <= tol_abs);         // NaN compares false -> reject
        if (BITS) {
            const float fd = (float)d, fm = (float)c_mis, fmatch = fd - fm;
            const bool rule = (fm < bp.pe_max * fd) && (c_mis == 0 || (float)c_close > bp.pm_min * fm) &&
                              (fmatch == 0.f || (float)c_msmall > bp.pw_min * fmatch) && (fabsf(st.mean_signed) <= bp.eps_max) &&
                              ((float)c_small >= bp.q_small_min * fd) && ((float)c_large <= bp.z_large_max * fd);
            vl_bit_stats bs;
            bs.n_exact = c_exact;
            bs.n_exp_mismatch = c_mis;
            bs.n_mismatch_close = c_close;
            bs.n_match_small = c_msmall;
            bs.n_small = c_small;
            bs.n_large = c_large;
            bs.mean_signed = st.mean_signed;
            bs.ok = rule ? 1u : 0u;
            if (bit_stats) bit_stats[row] = bs;
            ok = ok && rule;
        }
        if (ok_and) ok_and[row] = ok_and[row] & ok;
        if (ok_set) ok_set[row] = ok;
    }
}

void launch_compare(const float* h_hat, const void* committed, int hidden_dtype, int64_t rows, int d, float tol_rel,
                    float tol_abs, vl_tok_stats* stats, uint8_t* ok_and, uint8_t* ok_set, hipStream_t s,
                    const vl_bit_rule* rule, vl_bit_stats* bit_stats) {
    if (rows <= 0) return;
    dim3 grid((unsigned)((rows + 3) / 4));
    BitParams bp{};
    if (rule) {
        const long long tol = (long long)rule->e_m << rule->step_log2;
        bp = BitParams{rule->e_w, rule->q_small, rule->tau_large, (int)(tol > 0x7FFFFF ? 0x7FFFFF : tol), rule->pe_max,
                       rule->pm_min, rule->pw_min, rule->eps_max, rule->q_small_min, rule->z_large_max};
    }
#define VL_CMP(TC, BITS) compare_kernel<TC, BITS><<<grid, 256, 0, s>>>(h_hat, (const TC*)committed, rows, d, tol_rel, tol_abs, stats, \
                                                                        ok_and, ok_set, bp, bit_stats)
    if (hidden_dtype == VL_BF16) { if (rule) VL_CMP(bf16, true); else VL_CMP(bf16, false); }
    else { if (rule) VL_CMP(float, true); else VL_CMP(float, false); }
#undef VL_CMP
}

// ---------------------------------------------------------------- argmax + TokenMatch: one workgroup per row
__device__ __forceinline__ void take_better(float& bv, int& bi, float v, int i) {
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int vocab,
                                                     const int32_t* __restrict__ committed, float margin,
                                                     int32_t* __restrict__ out_argmax, float* __restrict__ out_gap,
                                                     uint8_t* __restrict__ out_ok) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int64_t row = blockIdx.x;
    const float* z = logits + row * (int64_t)vocab;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if ((vocab & 3) == 0) {
        const float4* z4 = (const float4*)z;
        const int n4 = vocab >> 2;
#pragma unroll 4
        for (int i = threadIdx.x; i < n4; i += 256) {
            const float4 t = z4[i];
            // ascending index within the lane, strict '>' keeps the lowest index among equals
            if (t.x > bv) { bv = t.x; bi = 4 * i; }
            if (t.y > bv) { bv = t.y; bi = 4 * i + 1; }
            if (t.z > bv) { bv = t.z; bi = 4 * i + 2; }
            if (t.w > bv) { bv = t.w; bi = 4 * i + 3; }
        }
    } else {
        for (int i = threadIdx.x; i < vocab; i += 256) {
            const float t = z[i];
            if (t > bv) { bv = t; bi = i; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, WAVE);
        const int oi = __shfl_xor(bi, o, WAVE);
        take_better(bv, bi, ov, oi);
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) take_better(bv, bi, sv[w], si[w]);
        if (bi == 0x7fffffff) bi = 0;                          // every logit NaN
        float gap = 0.f;
        uint8_t ok = 1;
        if (committed) {
            const int c = committed[row];
            if (c == -1) { gap = 0.f; ok = 1; }
            else if (c < 0 || c >= vocab) { gap = INFINITY; ok = 0; }
            else { gap = bv - z[c]; ok = (gap <= margin); }     // NaN compares false -> reject
        }
        if (out_argmax) out_argmax[row] = bi;
        if (out_gap) out_gap[row] = gap;
        if (out_ok) out_ok[row] = ok;
    }
}

void launch_argmax(const float* logits, int64_t rows, int vocab, const int32_t* committed, float margin,
                   int32_t* out_argmax, float* out_gap, uint8_t* out_ok, hipStream_t s) {
    if (rows <= 0) return;
    argmax_kernel<<<dim3((unsigned)rows), 256, 0, s>>>(logits, vocab, committed, margin, out_argmax, out_gap, out_ok);
}

// The same decision from per-part maxima: 16 tokens x 16 slices of the parts per workgroup; (maximum, lowest index) is a
// total order, so the result does not depend on how the parts are grouped.
__global__ __launch_bounds__(256) void argmax_reduce_kernel(ArgmaxParts ap, int n_parts, int64_t rows, int vocab,
                                                            const int32_t* __restrict__ committed, float margin,
                                                            int32_t* __restrict__ out_argmax, float* __restrict__ out_gap,
                                                            uint8_t* __restrict__ out_ok) {
    __shared__ float sv[16][16];
    __shared__ int si[16][16];
    const int t = threadIdx.x & 15, slice = threadIdx.x >> 4;
    const int64_t row = (int64_t)blockIdx.x * 16 + t;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if (row < rows)
        for (int p = slice; p < n_parts; p += 16) take_better(bv, bi, ap.pmax[p * ap.ld + row], ap.pidx[p * ap.ld + row]);
    sv[slice][t] = bv;
    si[slice][t] = bi;
    __syncthreads();
    if (slice != 0 || row >= rows) return;
#pragma unroll
    for (int w = 1; w < 16; ++w) take_better(bv, bi, sv[w][t], si[w][t]);
    if (bi == 0x7fffffff) bi = 0;                              // every logit NaN
    float gap = 0.f;
    uint8_t ok = 1;
    if (committed) {
        const int c = committed[row];
        if (c == -1) { gap = 0.f; ok = 1; }
        else if (c < 0 || c >= vocab) { gap = INFINITY; ok = 0; }
        else { gap = bv - ap.ztok[row]; ok = (gap <= margin); }     // NaN compares false -> reject
    }
    if (out_argmax) out_argmax[row] = bi;
    if (out_gap) out_gap[row] = gap;
    if (out_ok) out_ok[row] = ok;
}

void launch_argmax_reduce(const ArgmaxParts& parts, int64_t rows, int vocab, const int32_t* committed, float margin,
                          int32_t* out_argmax, float* out_gap, uint8_t* out_ok, hipStream_t s) {
    if (rows <= 0) return;
    argmax_reduce_kernel<<<dim3((unsigned)((rows + 15) / 16)), 256, 0, s>>>(parts, argmax_parts(vocab), rows, vocab, committed, margin,
                                                                           out_argmax, out_gap, out_ok);
}

// ---------------------------------------------------------------- flags + summary: one workgroup, fixed order
__global__ __launch_bounds__(1024) void finalize_kernel(const uint8_t* __restrict__ hid_ok, const uint8_t* __restrict__ tok_ok,
                                                        const vl_tok_stats* __restrict__ stats, int C, int64_t rows,
                                                        uint8_t* __restrict__ flags, DevSummary* __restrict__ out) {
    __shared__ unsigned long long s_rej[16], s_hid[16], s_tok[16];
    __shared__ float s_mr[16], s_ma[16];
    __shared__ double s_sum[16];
    unsigned long long rej = 0, hid = 0, tok = 0;
    for (int64_t n = threadIdx.x; n < rows; n += 1024) {
        const uint8_t h = hid_ok[n], t = tok_ok[n];
        const uint8_t f = h & t;
        flags[n] = f;
        rej += (f == 0);
        hid += (h == 0);
        tok += (t == 0);
    }
    float mr = 0.f, ma = 0.f;
    double sum = 0.0;
    const int64_t total = rows * (int64_t)C;
    for (int64_t i = threadIdx.x; i < total; i += 1024) {
        const vl_tok_stats st = stats[i];
        mr = fmaxf(mr, st.rel_l2);               // fmaxf ignores NaN, like a nan-max
        ma = fmaxf(ma, st.max_abs);
        sum += (double)st.mean_abs;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        rej += __shfl_xor(rej, o, WAVE);
        hid += __shfl_xor(hid, o, WAVE);
        tok += __shfl_xor(tok, o, WAVE);
        mr = fmaxf(mr, __shfl_xor(mr, o, WAVE));
        ma = fmaxf(ma, __shfl_xor(ma, o, WAVE));
        sum += __shfl_xor(sum, o, WAVE);
    }
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_rej[w] = rej; s_hid[w] = hid; s_tok[w] = tok; s_mr[w] = mr; s_ma[w] = ma; s_sum[w] = sum; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 16; ++i) {
            rej += s_rej[i]; hid += s_hid[i]; tok += s_tok[i];
            mr = fmaxf(mr, s_mr[i]); ma = fmaxf(ma, s_ma[i]); sum += s_sum[i];
        }
        out->n_rejected = rej;
        out->n_hidden_reject = hid;
        out->n_token_reject = tok;
        out->max_rel = mr;
        out->max_abs = ma;
        out->mean_mae = (float)(total > 0 ? sum / (double)total : 0.0);
    }
}

void launch_finalize(const uint8_t* hid_ok, const uint8_t* tok_ok, const vl_tok_stats* stats, int C, int64_t rows,
                     uint8_t* flags, DevSummary* out, hipStream_t s) {
    finalize_kernel<<<1, 1024, 0, s>>>(hid_ok, tok_ok, stats, C, rows, flags, out);
}

}  // namespace vl
