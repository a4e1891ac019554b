// Time chunks for full truncations.
//
// Chen's relation (Section 3, eq. 2) is associative, so a path may be cut into C consecutive chunks whose
// signatures S_1 .. S_C are computed independently (C times as many wavefronts for the sequential kernels) and
// multiplied afterwards:  S_{0,T} = S_1 (x) S_2 (x) .. (x) S_C,  where in the word basis
//     (a (x) b)(w) = sum_{k=0..n} a(w_1..w_k) b(w_{k+1}..w_n),   a(empty) = b(empty) = 1        (Section 2.1).
// The backward pass of chunk c needs the signature up to the end of the chunk, P_c = S_1 (x) .. (x) S_c, and the
// adjoint there, Abar_c(u) = sum_v grad(u v) Q_c(v) with Q_c = S_{c+1} (x) .. (x) S_C the signature of the rest
// of the path (Proposition 4.1 with the right factor taken at a chunk boundary).
//
// All arrays are [B][C][W] floats (W = d + d^2 + .. + d^N coefficients, levels concatenated, each row-major);
// d is a power of two so that prefixes and suffixes of a word index are shifts and masks.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.hpp"

namespace sig {
namespace {

struct Levels {
    int N;            // depth
    int lb;           // log2(d), >= 2
    int W;            // coefficients (a multiple of 4)
    int ls[14];       // ls[n] = index of the first word of length n, n = 1..N (multiples of 4); ls[N + 1] = W
};

typedef float f4 __attribute__((ext_vector_type(4)));

// Four consecutive coefficients (word length n, indices i .. i + 3 inside the level, i a multiple of 4) of a (x) b.
// The four words differ in their last letter only, so every prefix is shared and the suffixes are contiguous.
__device__ __forceinline__ f4 quad_product(const float* a, const float* b, const Levels& g, int n, int i)
{
    f4 acc = *(const f4*)(a + g.ls[n] + i) + *(const f4*)(b + g.ls[n] + i);
    for (int k = 1; k < n; ++k) {
        const int sh = g.lb * (n - k);
        const float av = a[g.ls[k] + (i >> sh)];
        const f4 bv = *(const f4*)(b + g.ls[n - k] + (i & ((1 << sh) - 1)));
        acc += av * bv;
    }
    return acc;
}

// out = a (x) b by the whole workgroup; out2 (may be null) receives a second copy.  Level by level, so that the
// level offsets and shifts are uniform.
__device__ __forceinline__ void tensor_product(const float* a, const float* b, float* out, float* out2, const Levels& g)
{
    for (int n = 1; n <= g.N; ++n) {
        const int quads = (g.ls[n + 1] - g.ls[n]) >> 2;
        for (int qd = threadIdx.x; qd < quads; qd += blockDim.x) {
            const f4 r = quad_product(a, b, g, n, 4 * qd);
            *(f4*)(out + g.ls[n] + 4 * qd) = r;
            if (out2) *(f4*)(out2 + g.ls[n] + 4 * qd) = r;
        }
    }
}

__device__ __forceinline__ void copy_row(const float* src, float* dst, float* dst2, int W)
{
    for (int o = 4 * threadIdx.x; o < W; o += 4 * blockDim.x) {
        const f4 v = *(const f4*)(src + o);
        *(f4*)(dst + o) = v;
        if (dst2) *(f4*)(dst2 + o) = v;
    }
}

// out(u) = gr(u) + sum_{m >= 1} sum_{|v| = m} gr(u v) q(v) for every word u, by the whole workgroup.  The words of
// one length k are spread over the workgroup, with blockDim / d^k threads (at most 64, at least 1) sharing the
// inner sums of a word; for a fixed m the terms of a word are contiguous in gr and in q.
// (k_only > 0: the words of that length alone, and with k_only == 1 also the copy of the longest words, so that a
// grid of N - 1 workgroups per row shares the work)
__device__ __forceinline__ void adjoint_contract(const float* gr, const float* q, float* __restrict__ out, const Levels& g,
                                                 int k_only = 0)
{
    const int N = g.N;
    if (k_only <= 1) copy_row(gr + g.ls[N], out + g.ls[N], nullptr, g.W - g.ls[N]);       // words of length N
    for (int k = 1; k < N; ++k) {
        if (k_only > 0 && k != k_only) continue;
        const int nk = g.ls[k + 1] - g.ls[k];                           // words of length k
        int tpw = (int)blockDim.x / nk;                                 // threads per word (power of two)
        tpw = tpw > 64 ? 64 : (tpw < 1 ? 1 : tpw);
        const int wpp = (int)blockDim.x / tpw;                          // words per pass
        const int t = threadIdx.x % tpw;
        for (int i0 = 0; i0 < nk; i0 += wpp) {
            const int i = i0 + threadIdx.x / tpw;
            float acc = 0.0f;
            if (i < nk)
                for (int m = 1; m <= N - k; ++m) {
                    const int cnt = 1 << (g.lb * m);
                    const float* src = gr + g.ls[k + m] + (i << (g.lb * m));
                    const float* qv = q + g.ls[m];
                    for (int v = t; v < cnt; v += tpw) acc = fmaf(src[v], qv[v], acc);
                }
            for (int off = tpw >> 1; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
            if (i < nk && t == 0) out[g.ls[k] + i] = gr[g.ls[k] + i] + acc;
        }
    }
}

// One workgroup per path.  Forward (Q == nullptr): coeffs_out[b] = S_1 (x) .. (x) S_C.  Backward: Pfx[c] =
// S_1 (x) .. (x) S_c for c < C and Pfx[C] = terminal[b] (the signature the caller kept), Q[c] = S_{c+1} (x) .. (x) S_C
// for c < C.  With LDS the running product and the next factor are staged in three rotating LDS buffers of W floats
// (small signatures); without, the operands are read from the global arrays written in earlier steps, which
// __syncthreads() makes visible inside the workgroup.  With LDS and Abar != nullptr the adjoints at the chunk
// boundaries, Abar[c](u) = sum_v grad(u v) Q[c](v), are formed here as well and Q is
// not written out; grad is read from global memory there (consecutive threads read consecutive coefficients).
template <bool LDS>
__global__ __launch_bounds__(1024) void chunk_scan_kernel(const float* __restrict__ Sc, float* Pfx, float* Q,
                                                          const float* __restrict__ terminal, float* coeffs_out,
                                                          const float* __restrict__ grad, float* Abar, int C, Levels g)
{
    extern __shared__ f4 smem4[];
    float* sm = (float*)smem4;
    const int64_t b = blockIdx.x;
    const int64_t W = g.W;
    const float* S = Sc + b * C * W;
    float* P = Pfx + b * C * W;
    const bool bwd = Q != nullptr;
    float* Qb = bwd ? Q + b * C * W : nullptr;
    if constexpr (LDS) {
        // gridDim.y == 2 (backward): workgroup 0 of a path does the prefix products, workgroup 1 the suffix products
        // and the adjoints, side by side; otherwise one workgroup does everything in turn
        const bool do_prefix = gridDim.y == 1 || blockIdx.y == 0;
        const bool do_suffix = bwd && (gridDim.y == 1 || blockIdx.y == 1);
        float* buf[3] = {sm, sm + W, sm + 2 * W};
        int cur = 0;
        if (do_prefix) {
            copy_row(S, buf[0], bwd ? P : nullptr, (int)W);
            const int lastp = bwd ? C - 2 : C - 1;
            for (int s = 1; s <= lastp; ++s) {
                const int nb = (cur + 1) % 3, no = (cur + 2) % 3;
                copy_row(S + (int64_t)s * W, buf[nb], nullptr, (int)W);
                __syncthreads();
                float* dst = (!bwd && s == C - 1) ? coeffs_out + b * W : (bwd ? P + (int64_t)s * W : nullptr);
                tensor_product(buf[cur], buf[nb], buf[no], dst, g);
                cur = no;
                __syncthreads();
            }
            if (bwd) copy_row(terminal + b * W, P + (int64_t)(C - 1) * W, nullptr, (int)W);
        }
        if (do_suffix) {
            const float* const gb = grad ? grad + b * W : nullptr;
            float* const Ab = Abar ? Abar + b * C * W : nullptr;
            if (Ab) copy_row(gb, Ab + (int64_t)(C - 1) * W, nullptr, (int)W);     // the last chunk's adjoint is grad
            // suffix products
            __syncthreads();
            copy_row(S + (int64_t)(C - 1) * W, buf[0], Ab ? nullptr : Qb + (int64_t)(C - 2) * W, (int)W);
            cur = 0;
            if (Ab) {
                __syncthreads();
                adjoint_contract(gb, buf[0], Ab + (int64_t)(C - 2) * W, g);
            }
            for (int q = C - 3; q >= 0; --q) {
                const int nb = (cur + 1) % 3, no = (cur + 2) % 3;
                copy_row(S + (int64_t)(q + 1) * W, buf[nb], nullptr, (int)W);
                __syncthreads();
                tensor_product(buf[nb], buf[cur], buf[no], Ab ? nullptr : Qb + (int64_t)q * W, g);
                cur = no;
                __syncthreads();
                if (Ab) adjoint_contract(gb, buf[cur], Ab + (int64_t)q * W, g);
            }
        }
    } else {
        // signatures too large for LDS: products in global memory; with gridDim.y == 2 (backward) workgroup 0 of a
        // path does the products from the left, workgroup 1 those from the right, side by side
        const bool do_prefix = gridDim.y == 1 || blockIdx.y == 0;
        const bool do_suffix = bwd && (gridDim.y == 1 || blockIdx.y == 1);
        if (do_prefix) {
            copy_row(S, P, nullptr, (int)W);
            if (bwd) copy_row(terminal + b * W, P + (int64_t)(C - 1) * W, nullptr, (int)W);
        }
        if (do_suffix) copy_row(S + (int64_t)(C - 1) * W, Qb + (int64_t)(C - 2) * W, nullptr, (int)W);
        const int last = bwd ? C - 2 : C - 1;
        for (int s = 1; s <= last; ++s) {
            __syncthreads();
            if (do_prefix) {
                float* dst = (!bwd && s == C - 1) ? coeffs_out + b * W : P + (int64_t)s * W;
                tensor_product(P + (int64_t)(s - 1) * W, S + (int64_t)s * W, dst, nullptr, g);
            }
            if (do_suffix) {
                const int q = C - 2 - s;              // >= 0 because s <= C - 2
                tensor_product(S + (int64_t)(q + 1) * W, Qb + (int64_t)(q + 1) * W, Qb + (int64_t)q * W, nullptr, g);
            }
        }
    }
}

// out[b] = a[b] (x) bfac[b] for every path, spread over the whole grid: blockIdx.y = path, blockIdx.x covers the
// quads of all levels.  Row strides are given in floats.
__global__ __launch_bounds__(256) void chunk_product_kernel(const float* __restrict__ a, int64_t a_stride,
                                                            const float* __restrict__ bfac, int64_t b_stride,
                                                            float* __restrict__ out, int64_t out_stride, Levels g)
{
    const int64_t b = blockIdx.y;
    const int o = 4 * (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (o >= g.W) return;
    int n = 1;
    while (o >= g.ls[n + 1]) ++n;
    *(f4*)(out + b * out_stride + o) = quad_product(a + b * a_stride, bfac + b * b_stride, g, n, o - g.ls[n]);
}

// dst[b] = src[b] for every path, rows of W floats (a multiple of 4) at the given strides
__global__ __launch_bounds__(256) void chunk_copy_rows_kernel(const float* __restrict__ src, int64_t src_stride, float* __restrict__ dst,
                                                              int64_t dst_stride, int W)
{
    const int o = 4 * (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (o >= W) return;
    *(f4*)(dst + (int64_t)blockIdx.y * dst_stride + o) = *(const f4*)(src + (int64_t)blockIdx.y * src_stride + o);
}

// coefficient of one word (length n, index i inside the level) of a (x) b
__device__ __forceinline__ float word_product(const float* a, const float* b, const Levels& g, int n, int i)
{
    float acc = a[g.ls[n] + i] + b[g.ls[n] + i];
    for (int k = 1; k < n; ++k) {
        const int sh = g.lb * (n - k);
        acc = fmaf(a[g.ls[k] + (i >> sh)], b[g.ls[n - k] + (i & ((1 << sh) - 1))], acc);
    }
    return acc;
}

// out[b] = a[b] (x) bfac[b] (x) c[b] in one pass (three time chunks, the usual count for long paths), without the
// intermediate array and its launch:
//     (a b c)(w) = c(w) + (a b)(w) + sum_{0 < l < n} (a b)(w_1..w_l) c(w_{l+1}..w_n),
//     (a b)(w)   = a(w) + b(w)     + sum_{0 < k < n} a(w_1..w_k) b(w_{k+1}..w_n).
// A workgroup takes 1,024 consecutive words of one length n (blockIdx.x runs over the lengths, each padded to whole
// workgroups).  Their prefixes of length l are the 1,024 / d^(n-l) (at least one) consecutive words of that length,
// so a(prefix) and (a b)(prefix) are computed once per workgroup into LDS; what a thread then reads per quad is
// the three quads of w and, per cut, one suffix quad of b and one of c.
constexpr int kProduct3Prefixes = 384;             // 256 + 64 + 16 + 4 + 1 + ... for d = 4; fewer for larger d

__host__ __device__ inline int product3_blocks(const Levels& g, int n) { return ((g.ls[n + 1] - g.ls[n]) / 4 + 255) / 256; }

__global__ __launch_bounds__(256) void chunk_product3_kernel(const float* __restrict__ a, const float* __restrict__ bfac,
                                                             const float* __restrict__ c, int64_t in_stride,
                                                             float* __restrict__ out, int64_t out_stride, Levels g)
{
    __shared__ float sA[kProduct3Prefixes], sAB[kProduct3Prefixes];
    const int64_t b = blockIdx.y;
    int blk = (int)blockIdx.x, n = 1;
    while (n < g.N && blk >= product3_blocks(g, n)) { blk -= product3_blocks(g, n); ++n; }
    const int words = g.ls[n + 1] - g.ls[n];
    const int i0 = blk * 1024;                         // first word of the workgroup inside its length
    const float* pa = a + b * in_stride;
    const float* pb = bfac + b * in_stride;
    const float* pc = c + b * in_stride;
    // prefixes of length l = 1 .. n - 1 of the words i0 .. i0 + 1023: cnt_l consecutive words from p0_l on
    int off = 0;
    for (int l = 1; l < n; ++l) {
        const int sh = g.lb * (n - l);
        const int p0 = i0 >> sh;
        const int cnt = (1024 >> sh) > 0 ? (1024 >> sh) : 1;
        const int have = g.ls[l + 1] - g.ls[l];
        for (int t = threadIdx.x; t < cnt; t += blockDim.x)
            if (p0 + t < have) {
                sA[off + t] = pa[g.ls[l] + p0 + t];
                sAB[off + t] = word_product(pa, pb, g, l, p0 + t);
            }
        off += cnt;
    }
    __syncthreads();
    const int i = i0 + 4 * (int)threadIdx.x;
    if (i >= words) return;
    const int o = g.ls[n] + i;
    f4 acc = (*(const f4*)(pa + o) + *(const f4*)(pb + o)) + *(const f4*)(pc + o);
    off = 0;
    for (int l = 1; l < n; ++l) {
        const int sh = g.lb * (n - l);
        const int pi = off + (i >> sh) - (i0 >> sh);
        const int suffix = g.ls[n - l] + (i & ((1 << sh) - 1));
        acc += sA[pi] * *(const f4*)(pb + suffix);
        acc += sAB[pi] * *(const f4*)(pc + suffix);
        off += (1024 >> sh) > 0 ? (1024 >> sh) : 1;
    }
    *(f4*)(out + b * out_stride + o) = acc;
}

// One workgroup per (path, chunk): Abar[b][c](u) = grad[b](u) + sum_{m >= 1} sum_{|v| = m} grad[b](u v) Q[b][c](v);
// the last chunk's adjoint is grad itself.  The words of one length k are spread over the whole workgroup, with
// blockDim / d^k threads (at most 64, at least 1) sharing the inner sums of a word; for a fixed m the terms of a
// word are contiguous in grad and in Q.
template <bool LDS>
__global__ __launch_bounds__(512) void chunk_adjoint_kernel(const float* __restrict__ grad, const float* __restrict__ Q,
                                                            float* __restrict__ Abar, int C, bool skip_last, Levels g)
{
    extern __shared__ f4 smem4[];
    float* sm = (float*)smem4;
    const int64_t row = blockIdx.x;
    const int64_t b = row / C;
    const int c = (int)(row - b * C);
    const int W = g.W;
    const float* gr = grad + b * W;
    // without the rows of the last chunk the array is [B][C - 1][W]
    float* out = Abar + (skip_last ? row - b : row) * W;
    if (c == C - 1) {
        if (!skip_last && blockIdx.y == 0) copy_row(gr, out, nullptr, W);
        return;
    }
    const float* q = Q + row * W;
    if constexpr (LDS) {
        copy_row(gr, sm, nullptr, W);
        copy_row(q, sm + W, nullptr, W);
        __syncthreads();
        gr = sm;
        q = sm + W;
    }
    // large signatures: one workgroup per (row, word length), their sums read global memory and are bound by latency
    adjoint_contract(gr, q, out, g, gridDim.y > 1 ? (int)blockIdx.y + 1 : 0);
}

// The same sums for large signatures, one workgroup per (path, chunk, first letter a): every word u that begins with a
// gets Abar(u) = grad(u) + sum_v grad(u v) Q(v).  The words u v all begin with a too, so workgroups share no output,
// and what a workgroup reads - the gradients of the words a v and Q(v) for |v| < N, 2 (d + .. + d^(N-1)) floats - is
// staged in LDS once: sg[ls[m] + v] = grad(a v), sq[ls[m] + v] = Q(v) for |v| = m.  All 512 threads work on one word
// length at a time and split the sums of a word between 512 / (words of that length) of them (whole wavefronts add
// up through LDS), so that short words, whose sums run over thousands of terms, take as few rounds as long ones.
__global__ __launch_bounds__(512) void chunk_adjoint_subtree_kernel(const float* __restrict__ grad, const float* __restrict__ Q,
                                                                    float* __restrict__ Abar, int C, Levels g)
{
    extern __shared__ f4 smem4[];
    __shared__ float red[8];
    const int64_t row = blockIdx.x;
    const int64_t b = row / C;
    if ((int)(row - b * C) == C - 1) return;             // the last chunk's adjoint is the gradient itself
    const int a = (int)blockIdx.y;
    const int N = g.N, W = g.W, lb = g.lb;
    const int below = g.ls[N];                           // words shorter than N
    float* sq = (float*)smem4;
    float* sg = sq + below;
    const float* gr = grad + b * W;
    const float* q = Q + row * W;
    float* out = Abar + (row - b) * W;                   // [B][C - 1][W]: the last chunk has no row
    const int tid = (int)threadIdx.x, nthr = (int)blockDim.x;
    for (int m = 1; m < N; ++m) {
        const int cnt = 1 << (lb * m);
        const float* src = gr + g.ls[m + 1] + (int64_t)a * cnt;      // the words a v, |v| = m
        for (int v = tid; v < cnt; v += nthr) {
            sq[g.ls[m] + v] = q[g.ls[m] + v];
            sg[g.ls[m] + v] = src[v];
        }
    }
    {
        const int cnt = 1 << (lb * (N - 1));             // words of length N that begin with a: copied
        const float* src = sg + g.ls[N - 1];
        float* dst = out + g.ls[N] + a * cnt;
        __syncthreads();
        for (int o = 4 * tid; o < cnt; o += 4 * nthr) *(f4*)(dst + o) = *(const f4*)(src + o);
    }
    for (int k = 1; k < N; ++k) {
        const int nk = 1 << (lb * (k - 1));              // words of length k that begin with a: u = a u', |u'| = k - 1
        int tpw = nthr / nk;                             // threads per word (a power of two)
        tpw = tpw < 1 ? 1 : tpw;
        const int wpp = nthr / tpw;                      // words per pass
        const int t = tid % tpw;
        for (int i0 = 0; i0 < nk; i0 += wpp) {
            const int iw = i0 + tid / tpw;               // u' inside its length
            float acc = 0.0f;
            if (iw < nk)
                for (int m = 1; m <= N - k; ++m) {
                    const int cnt = 1 << (lb * m);
                    const float* src = sg + g.ls[k - 1 + m] + (iw << (lb * m));   // the words a u' v
                    const float* qv = sq + g.ls[m];
                    for (int v = t; v < cnt; v += tpw) acc = fmaf(src[v], qv[v], acc);
                }
            const int within = tpw < 64 ? tpw : 64;
            for (int off = within >> 1; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
            if (tpw > 64) {                              // a word's threads span tpw / 64 consecutive wavefronts
                __syncthreads();
                if ((tid & 63) == 0) red[tid >> 6] = acc;
                __syncthreads();
                if (t == 0) {
                    acc = 0.0f;
                    for (int wv = 0; wv < tpw / 64; ++wv) acc += red[(tid >> 6) + wv];
                }
            }
            if (iw < nk && t == 0) {
                const float own = k == 1 ? gr[g.ls[1] + a] : sg[g.ls[k - 1] + iw];
                out[g.ls[k] + a * nk + iw] = own + acc;
            }
        }
    }
}

constexpr size_t kMaxChunkLds = 96 * 1024;       // three signatures of up to 8,192 coefficients

bool make_levels(int d, int depth, Levels& g)
{
    if (d < 4 || (d & (d - 1)) != 0 || depth < 2 || depth > 12) return false;
    g.N = depth;
    g.lb = 0;
    while ((1 << g.lb) < d) ++g.lb;
    if (g.lb * depth > 30) return false;
    int64_t off = 0;
    g.ls[0] = 0;
    for (int n = 1; n <= depth; ++n) {
        g.ls[n] = (int)off;
        off += (int64_t)1 << (g.lb * n);
    }
    if (off > 0x7fffffff) return false;
    g.ls[depth + 1] = (int)off;
    g.W = (int)off;
    return true;
}

}  // namespace

bool chunking_available(int d, int depth)
{
    Levels g;
    return make_levels(d, depth, g);
}

hipError_t chunk_scan(int d, int depth, const float* Sc, float* Pfx, float* Q, const float* terminal, float* coeffs_out,
                      const float* grad, float* Abar, int64_t B, int C, bool* adjoints_done, hipStream_t stream)
{
    if (adjoints_done) *adjoints_done = false;
    Levels g;
    if (!make_levels(d, depth, g) || C < 2 || B < 1 || B > 0x7fffffff) return hipErrorInvalidValue;
    if ((Q != nullptr) != (terminal != nullptr) || (Q == nullptr) == (coeffs_out == nullptr)) return hipErrorInvalidValue;
    const bool fuse = Q != nullptr && grad != nullptr && Abar != nullptr;
    const size_t lds = 3 * (size_t)g.W * sizeof(float);
    if (lds <= kMaxChunkLds) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&chunk_scan_kernel<true>), (int)kMaxChunkLds);
        if (e != hipSuccess) return e;
        chunk_scan_kernel<true><<<dim3((unsigned)B, fuse ? 2 : 1), 1024, lds, stream>>>(
            Sc, Pfx, Q, terminal, coeffs_out, fuse ? grad : nullptr, fuse ? Abar : nullptr, C, g);
        if (fuse && adjoints_done) *adjoints_done = true;
    } else if (Q == nullptr && B <= 65535) {
        // forward with large signatures: one grid-wide product per chunk boundary
        const int64_t W = g.W;
        const dim3 grid((unsigned)((W / 4 + 255) / 256), (unsigned)B);
        if (C == 3) {
            unsigned blocks = 0;
            for (int n = 1; n <= g.N; ++n) blocks += (unsigned)product3_blocks(g, n);
            chunk_product3_kernel<<<dim3(blocks, (unsigned)B), 256, 0, stream>>>(Sc, Sc + W, Sc + 2 * (int64_t)W, (int64_t)C * W,
                                                                               coeffs_out, W, g);
            return hipGetLastError();
        }
        const float* acc = Sc;                       // S_1 of every path, row stride C W
        int64_t acc_stride = (int64_t)C * W;
        for (int s = 1; s < C; ++s) {
            float* dst = s == C - 1 ? coeffs_out : Pfx + (int64_t)s * W;
            const int64_t dst_stride = s == C - 1 ? W : (int64_t)C * W;
            chunk_product_kernel<<<grid, 256, 0, stream>>>(acc, acc_stride, Sc + (int64_t)s * W, (int64_t)C * W, dst,
                                                           dst_stride, g);
            acc = dst;
            acc_stride = dst_stride;
        }
    } else if (Q != nullptr && coeffs_out == nullptr && B <= 64 && g.W % 4 == 0) {
        // backward with large signatures and few paths: a workgroup or two per path would leave the chip idle, so every
        // product is spread over the whole grid (a launch per chunk boundary and direction)
        const int64_t W = g.W, row = (int64_t)C * W;
        const dim3 grid((unsigned)((W / 4 + 255) / 256), (unsigned)B);
        chunk_copy_rows_kernel<<<grid, 256, 0, stream>>>(Sc, row, Pfx, row, (int)W);
        chunk_copy_rows_kernel<<<grid, 256, 0, stream>>>(terminal, W, Pfx + (int64_t)(C - 1) * W, row, (int)W);
        chunk_copy_rows_kernel<<<grid, 256, 0, stream>>>(Sc + (int64_t)(C - 1) * W, row, Q + (int64_t)(C - 2) * W, row, (int)W);
        for (int s = 1; s <= C - 2; ++s) {
            chunk_product_kernel<<<grid, 256, 0, stream>>>(Pfx + (int64_t)(s - 1) * W, row, Sc + (int64_t)s * W, row,
                                                           Pfx + (int64_t)s * W, row, g);
            const int q = C - 2 - s;
            chunk_product_kernel<<<grid, 256, 0, stream>>>(Sc + (int64_t)(q + 1) * W, row, Q + (int64_t)(q + 1) * W, row,
                                                           Q + (int64_t)q * W, row, g);
        }
    } else {
        chunk_scan_kernel<false><<<dim3((unsigned)B, Q != nullptr ? 2 : 1), 1024, 0, stream>>>(Sc, Pfx, Q, terminal, coeffs_out, nullptr,
                                                                                          nullptr, C, g);
    }
    return hipGetLastError();
}

hipError_t chunk_adjoint(int d, int depth, const float* grad, const float* Q, float* Abar, int64_t B, int C, bool skip_last,
                         hipStream_t stream)
{
    Levels g;
    if (!make_levels(d, depth, g) || C < 2 || B < 1 || B * C > 0x7fffffff) return hipErrorInvalidValue;
    const size_t lds = 2 * (size_t)g.W * sizeof(float);
    if (lds <= 64 * 1024) chunk_adjoint_kernel<true><<<(unsigned)(B * C), 512, lds, stream>>>(grad, Q, Abar, C, skip_last, g);
    else if (skip_last && g.lb * (g.N - 1) >= 2 && 2 * (size_t)g.ls[g.N] * sizeof(float) <= 64 * 1024)
        chunk_adjoint_subtree_kernel<<<dim3((unsigned)(B * C), 1u << g.lb), 512, 2 * (size_t)g.ls[g.N] * sizeof(float), stream>>>(
            grad, Q, Abar, C, g);
    else chunk_adjoint_kernel<false><<<dim3((unsigned)(B * C), (unsigned)(g.N - 1)), 512, 0, stream>>>(grad, Q, Abar, C, skip_last, g);
    return hipGetLastError();
}

}  // namespace sig
