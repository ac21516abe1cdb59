// Merkle commitment of hidden states (Section 5.6 "Commitment Submission": root = MerkleRoot(S) over a canonical
// serialization with scalar elements as leaves; Section 7: canonical float32, SHA-256).
//
//   leaf j      = SHA-256(the 4 little-endian bytes of element j as float32)      (a bf16 state is upcast exactly)
//   inner node  = SHA-256(left digest || right digest)
//   a node without a right neighbour at its level moves up unchanged
//
// Pure integer ALU work: d leaf compressions and 2 (d - 1) node compressions per state row (a 64-byte message takes a
// second, constant padding block), each 64 rounds.  One workgroup per row: thread t streams the leaves of its aligned
// block of 2^s leaves through a binary-counter stack (LDS, s + 1 digests per thread) and ends with the digest of
// that subtree; the remaining <= 256 digests are reduced level by level in LDS.  The round constants are derived at
// compile time from their definition (fractional parts of the cube / square roots of the first primes).
#include "common.h"
#include "kernels.h"

namespace vl {

// ---------------------------------------------------------------- SHA-256 constants from their definition
namespace sha {
typedef unsigned __int128 u128;
constexpr bool is_prime(int n) {
    for (int i = 2; i * i <= n; ++i)
        if (n % i == 0) return false;
    return n >= 2;
}
constexpr int nth_prime(int k) {                                // k = 0 -> 2
    int n = 1;
    for (int seen = -1; seen < k;) {
        ++n;
        if (is_prime(n)) ++seen;
    }
    return n;
}
// floor(frac(p^(1/R)) * 2^32) = floor((p * 2^(32 R))^(1/R)) mod 2^32, by bisection on integers
constexpr uint32_t frac_root(int p, int R) {
    const u128 target = (u128)p << (32 * R);
    uint64_t lo = 0, hi = (uint64_t)1 << 36;
    while (hi - lo > 1) {
        const uint64_t mid = lo + (hi - lo) / 2;
        u128 pw = 1;
        for (int i = 0; i < R; ++i) pw *= mid;
        if (pw <= target) lo = mid; else hi = mid;
    }
    return (uint32_t)lo;
}
struct Tables { uint32_t k[64]; uint32_t h[8]; };
constexpr Tables make_tables() {
    Tables t{};
    for (int i = 0; i < 64; ++i) t.k[i] = frac_root(nth_prime(i), 3);
    for (int i = 0; i < 8; ++i) t.h[i] = frac_root(nth_prime(i), 2);
    return t;
}
constexpr Tables T = make_tables();
static_assert(T.k[0] == 0x428a2f98u && T.k[63] == 0xc67178f2u && T.h[0] == 0x6a09e667u && T.h[7] == 0x5be0cd19u,
              "SHA-256 constants");

__device__ __forceinline__ uint32_t rotr(uint32_t x, int n) { return __builtin_rotateright32(x, n); }

// One compression: st += compress(st, w).  Fully unrolled, so a constant message word folds into its round.
__device__ __forceinline__ void compress(uint32_t (&st)[8], uint32_t (&w)[16]) {
    uint32_t a = st[0], b = st[1], c = st[2], d = st[3], e = st[4], f = st[5], g = st[6], h = st[7];
#pragma unroll
    for (int t = 0; t < 64; ++t) {
        if (t >= 16) {
            const uint32_t w15 = w[(t - 15) & 15], w2 = w[(t - 2) & 15];
            const uint32_t s0 = rotr(w15, 7) ^ rotr(w15, 18) ^ (w15 >> 3);
            const uint32_t s1 = rotr(w2, 17) ^ rotr(w2, 19) ^ (w2 >> 10);
            w[t & 15] = w[t & 15] + s0 + w[(t - 7) & 15] + s1;
        }
        const uint32_t S1 = rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25);
        const uint32_t ch = (e & f) ^ (~e & g);
        const uint32_t t1 = h + S1 + ch + T.k[t] + w[t & 15];
        const uint32_t S0 = rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22);
        const uint32_t mj = (a & b) ^ (a & c) ^ (b & c);
        const uint32_t t2 = S0 + mj;
        h = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    st[0] += a; st[1] += b; st[2] += c; st[3] += d; st[4] += e; st[5] += f; st[6] += g; st[7] += h;
}

__device__ __forceinline__ void init(uint32_t (&st)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) st[i] = T.h[i];
}

// digest of the 4-byte message holding `bits` in little-endian order
__device__ __forceinline__ void leaf(uint32_t bits, uint32_t (&out)[8]) {
    uint32_t w[16];
    w[0] = __builtin_bswap32(bits);                             // message bytes b0 b1 b2 b3 form the big-endian word
    w[1] = 0x80000000u;
#pragma unroll
    for (int i = 2; i < 15; ++i) w[i] = 0;
    w[15] = 32;                                                 // message length in bits
    init(out);
    compress(out, w);
}

// digest of the 64-byte message left || right
__device__ __forceinline__ void node(const uint32_t (&l)[8], const uint32_t (&r)[8], uint32_t (&out)[8]) {
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) { w[i] = l[i]; w[8 + i] = r[i]; }
    init(out);
    compress(out, w);
    w[0] = 0x80000000u;
#pragma unroll
    for (int i = 1; i < 15; ++i) w[i] = 0;
    w[15] = 512;
    compress(out, w);
}
}  // namespace sha

constexpr int MK_THREADS = 256;
constexpr int MK_MAX_S = 6;                                     // up to 2^6 leaves per thread: d_model <= 16384

template <typename T> __device__ __forceinline__ uint32_t f32_bits(const T* p);
template <> __device__ __forceinline__ uint32_t f32_bits<float>(const float* p) { return __float_as_uint(*p); }
template <> __device__ __forceinline__ uint32_t f32_bits<bf16>(const bf16* p) { return ((uint32_t)*(const uint16_t*)p) << 16; }

// ---------------------------------------------------------------- roots: one workgroup per state row
template <typename T>
__global__ __launch_bounds__(MK_THREADS) void merkle_root_kernel(const T* __restrict__ states, int d, int s,
                                                                 uint8_t* __restrict__ roots) {
    __shared__ uint32_t stack[MK_MAX_S + 1][8][MK_THREADS];     // [level][word][thread]: conflict-free
    __shared__ uint32_t nodes[2][MK_THREADS][8];
    const int tid = threadIdx.x;
    const T* row = states + (int64_t)blockIdx.x * d;
    const int bl = 1 << s;
    const int nb = (d + bl - 1) >> s;                           // threads that own leaves (<= 256)
    if (tid < nb) {
        const int j0 = tid << s, j1 = min(j0 + bl, d);
        uint32_t has = 0;                                       // bit l: the stack holds a subtree of 2^l leaves
        for (int j = j0; j < j1; ++j) {
            uint32_t cur[8];
            sha::leaf(f32_bits<T>(row + j), cur);
            int lvl = 0;
            while (has & (1u << lvl)) {
                uint32_t left[8], out[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) left[i] = stack[lvl][i][tid];
                sha::node(left, cur, out);
#pragma unroll
                for (int i = 0; i < 8; ++i) cur[i] = out[i];
                has &= ~(1u << lvl);
                ++lvl;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) stack[lvl][i][tid] = cur[i];
            has |= 1u << lvl;
        }
        // fold what is left (only a ragged last block leaves more than one entry): lower levels lie to the right
        uint32_t cur[8];
        bool have = false;
        for (int lvl = 0; lvl <= s; ++lvl) {
            if (!(has & (1u << lvl))) continue;
            uint32_t left[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) left[i] = stack[lvl][i][tid];
            if (!have) {
#pragma unroll
                for (int i = 0; i < 8; ++i) cur[i] = left[i];
                have = true;
            } else {
                uint32_t out[8];
                sha::node(left, cur, out);
#pragma unroll
                for (int i = 0; i < 8; ++i) cur[i] = out[i];
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) nodes[0][tid][i] = cur[i];
    }
    __syncthreads();
    int cnt = nb, src = 0;
    while (cnt > 1) {                                           // uniform
        const int half = cnt >> 1;
        if (tid < half) {
            uint32_t l[8], r[8], out[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) { l[i] = nodes[src][2 * tid][i]; r[i] = nodes[src][2 * tid + 1][i]; }
            sha::node(l, r, out);
#pragma unroll
            for (int i = 0; i < 8; ++i) nodes[src ^ 1][tid][i] = out[i];
        } else if (tid == half && (cnt & 1)) {
#pragma unroll
            for (int i = 0; i < 8; ++i) nodes[src ^ 1][tid][i] = nodes[src][cnt - 1][i];
        }
        __syncthreads();
        cnt = (cnt + 1) >> 1;
        src ^= 1;
    }
    if (tid < 8) {
        const uint32_t v = nodes[src][0][tid];
        uint8_t* o = roots + (int64_t)blockIdx.x * 32 + 4 * tid;
        o[0] = (uint8_t)(v >> 24); o[1] = (uint8_t)(v >> 16); o[2] = (uint8_t)(v >> 8); o[3] = (uint8_t)v;
    }
}

// ---------------------------------------------------------------- openings: one workgroup per disclosed element
// Plain level-by-level tree in a global scratch area (2 x d digests per workgroup); at every level the sibling of the
// path node, if there is one, is copied out.  Openings are few, so nothing here is tuned.
template <typename T>
__global__ __launch_bounds__(MK_THREADS) void merkle_open_kernel(const T* __restrict__ states, int d, int depth,
                                                                 const int32_t* __restrict__ sel_row,
                                                                 const int32_t* __restrict__ sel_idx,
                                                                 uint32_t* __restrict__ scratch, uint8_t* __restrict__ paths,
                                                                 float* __restrict__ values) {
    const int tid = threadIdx.x, q = blockIdx.x;
    const T* row = states + (int64_t)sel_row[q] * d;
    uint32_t* lev[2] = {scratch + (int64_t)q * 2 * d * 8, scratch + ((int64_t)q * 2 + 1) * d * 8};
    for (int j = tid; j < d; j += MK_THREADS) {
        uint32_t h[8];
        sha::leaf(f32_bits<T>(row + j), h);
#pragma unroll
        for (int i = 0; i < 8; ++i) lev[0][(int64_t)j * 8 + i] = h[i];
    }
    __syncthreads();
    int n = d, idx = sel_idx[q], src = 0, k = 0;
    if (tid == 0 && values) values[q] = __uint_as_float(f32_bits<T>(row + idx));
    while (n > 1) {                                             // uniform
        const int sib = idx ^ 1;
        if (sib < n) {
            if (tid < 8) {
                const uint32_t v = lev[src][(int64_t)sib * 8 + tid];
                uint8_t* o = paths + ((int64_t)q * depth + k) * 32 + 4 * tid;
                o[0] = (uint8_t)(v >> 24); o[1] = (uint8_t)(v >> 16); o[2] = (uint8_t)(v >> 8); o[3] = (uint8_t)v;
            }
            ++k;
        }
        const int half = n >> 1;
        for (int p = tid; p < half; p += MK_THREADS) {
            uint32_t l[8], r[8], out[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) { l[i] = lev[src][(int64_t)(2 * p) * 8 + i]; r[i] = lev[src][(int64_t)(2 * p + 1) * 8 + i]; }
            sha::node(l, r, out);
#pragma unroll
            for (int i = 0; i < 8; ++i) lev[src ^ 1][(int64_t)p * 8 + i] = out[i];
        }
        if ((n & 1) && tid < 8) lev[src ^ 1][(int64_t)half * 8 + tid] = lev[src][(int64_t)(n - 1) * 8 + tid];
        __syncthreads();
        n = (n + 1) >> 1;
        idx >>= 1;
        src ^= 1;
    }
    for (int e = k * 32 + tid; e < depth * 32; e += MK_THREADS) paths[(int64_t)q * depth * 32 + e] = 0;   // unused entries
}

int merkle_depth(int d) {
    int depth = 0;
    while ((1 << depth) < d) ++depth;
    return depth;
}

void launch_merkle_roots(const void* states, int dtype, int64_t rows, int d, uint8_t* roots, hipStream_t s) {
    if (rows <= 0) return;
    int sl = 0;
    while (((d + (1 << sl) - 1) >> sl) > MK_THREADS) ++sl;      // smallest block size that fits the row into 256 threads
    if (dtype == VL_BF16)
        merkle_root_kernel<bf16><<<dim3((unsigned)rows), MK_THREADS, 0, s>>>((const bf16*)states, d, sl, roots);
    else
        merkle_root_kernel<float><<<dim3((unsigned)rows), MK_THREADS, 0, s>>>((const float*)states, d, sl, roots);
}

void launch_merkle_open(const void* states, int dtype, int d, const int32_t* sel_row, const int32_t* sel_idx, int count,
                        uint32_t* scratch, uint8_t* paths, float* values, hipStream_t s) {
    if (count <= 0) return;
    const int depth = merkle_depth(d);
    if (dtype == VL_BF16)
        merkle_open_kernel<bf16><<<dim3((unsigned)count), MK_THREADS, 0, s>>>((const bf16*)states, d, depth, sel_row, sel_idx,
                                                                            scratch, paths, values);
    else
        merkle_open_kernel<float><<<dim3((unsigned)count), MK_THREADS, 0, s>>>((const float*)states, d, depth, sel_row, sel_idx,
                                                                             scratch, paths, values);
}

}  // namespace vl
