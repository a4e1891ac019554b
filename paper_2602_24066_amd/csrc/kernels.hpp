// Launch interface between the C ABI (api.cpp) and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <set>
#include <utility>

#include "wordset.hpp"

namespace sig {

// Raises a kernel's dynamic-LDS limit (needed above 64 KB) once per (device, kernel).  Safe for concurrent callers.
inline hipError_t ensure_dynamic_lds(const void* kernel, int bytes)
{
    static std::mutex m;
    static std::set<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(m);
    if (done.count({dev, kernel})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.insert({dev, kernel});
    return e;
}

struct GenericArgs {
    const UnitDesc* units = nullptr;      // device
    const uint32_t* ops = nullptr;        // device
    const int32_t* slot_word = nullptr;   // device
    int64_t n_units = 0;
    int max_slots = 0;
    const float* path = nullptr;          // device [B, P, d]
    int64_t B = 0, P = 0;
    int d = 0;
    int64_t nW = 0;
    float* coeffs = nullptr;              // forward output
    const float* coeffs_in = nullptr;     // backward inputs
    const float* grad_coeffs = nullptr;
    float* gdx = nullptr;                 // backward: [B, L, d] accumulation buffer (zeroed by the caller)
    int tile_steps = 1;
};

size_t generic_bwd_lds_bytes(int d, int max_slots, int tile_steps);
hipError_t generic_forward(const GenericArgs& a, int max_len, hipStream_t stream);
hipError_t generic_backward(const GenericArgs& a, int max_len, hipStream_t stream);


hipError_t fill_zero(float* p, int64_t n, hipStream_t stream);
hipError_t leadlag(const float* path, int64_t B, int64_t P, int d, float* out, hipStream_t stream);            // out [B, 2P-1, 2d]
hipError_t leadlag_backward(const float* gout, int64_t B, int64_t P, int d, float* gpath, hipStream_t stream);
// windows: (path, window) pairs as paths of n_sub points each, and the adjoint of that gather
hipError_t window_gather(const float* path, int64_t B, int64_t P, int d, const int64_t* win, int64_t K, int64_t n_sub, float* sub,
                         hipStream_t stream);
hipError_t window_scatter(const float* gsub, int64_t B, int64_t P, int d, const int64_t* win, int64_t K, int64_t n_sub,
                          float* gpath, hipStream_t stream);
// log-signature coordinates from signature coefficients, and the adjoint (gcoeffs overwritten)
hipError_t logsig_forward(const float* coeffs, int64_t B, int64_t nW, const int32_t* lyn_len, const int32_t* lyn_sub, int64_t n_lyn,
                          int stride, int depth, float* out, hipStream_t stream);
hipError_t logsig_backward(const float* coeffs, const float* glog, int64_t B, int64_t nW, const int32_t* lyn_len,
                           const int32_t* lyn_sub, int64_t n_lyn, int stride, int depth, int n_pairs, const int32_t* inv_off,
                           const int32_t* inv, float* part /*[B, n_lyn, n_pairs]*/, float* gcoeffs, bool two_kernels,
                           hipStream_t stream);
// Device memory of the entry point that allocates nothing: address of this device's copy of the library's static
// scratch array (SIG_STATIC_SCRATCH_BYTES bytes, 256-byte aligned), looked up once per device.
hipError_t static_scratch(void** ptr);
hipError_t fma_probe(float* out, int blocks, int iters, hipStream_t stream);   // out: blocks * 256 floats
hipError_t issue_probe(float* out, int blocks, int iters, int mode, hipStream_t stream);   // out: blocks * 256 floats
hipError_t grad_points(const float* gdx, int64_t B, int64_t P, int d, float* grad_path, hipStream_t stream);

// Window list of a launch (signatures over windows): K windows per path, window k between the points win[2 k] and
// win[2 k + 1] (device array, clamped to the path by the kernels), at most max_len segments; win == nullptr: no windows.
// A list without windows but with K > 1 cuts every path into K time chunks of max_len segments (the last one shorter):
// the rows of a launch over all (path, chunk) pairs.
struct WindowList {
    const int64_t* win = nullptr;
    int64_t K = 0;
    int64_t max_len = 0;
    __host__ __device__ bool several_rows() const { return win != nullptr || K > 1; }   // rows of one path share points
    __host__ __device__ int64_t rows_per_path() const { return several_rows() ? K : 1; }
};

// Increments of B paths (or, with a window list, of the B * K windows of the paths: one row per (path, window) pair,
// read straight from the path), differenced and transposed for the specialised kernels; Lpad: padded segments per row.
// zeroed: nullptr, or an array of the layout of dxT that the kernel clears on the way (the increment gradients).
hipError_t increments_transposed(const float* path, int64_t B, int64_t P, int d, int64_t Lpad, float* dxT, float* zeroed,
                                 hipStream_t stream, const WindowList& wl = WindowList());
// chain rule from increment gradients in the layout of increments_transposed to grad_path [B][P][d]; with a window list
// the rows are windows and their gradients are added into grad_path (zeroed by the caller)
hipError_t grad_points_transposed(const float* g, int64_t B, int64_t P, int d, int64_t Lpad, float* grad_path, hipStream_t stream,
                                  const WindowList& wl = WindowList());

// Time chunks for word sets closed under prefixes and suffixes (kernels_words.hip).  Device tables of such a set:
struct WordTables {
    const uint32_t* prod_pairs = nullptr;   // terms of the product by word, see WordSet::prod_pairs
    const uint32_t* adj_pairs = nullptr;    // the same terms by prefix, see WordSet::adj_pairs
    const uint32_t* adj_key = nullptr;      // the prefix of every entry of adj_pairs (W: padding)
    int adj_groups = 0;                     // entries of adj_pairs / 256
    int32_t level_start[16] = {};           // [N + 2]
    int32_t tail_off[16] = {};              // [N + 2]
    int N = 0;                              // longest word (<= 14)
    int W = 0;                              // number of words (<= 65,535)
};
size_t words_scan_lds_bytes(int64_t W);
// S [B][C][W] chunk signatures.  Forward scan: rows[b][c] = S_0 (x) .. (x) S_c (if rows), last[b] = the product of all
// (if last).  Reverse scan: rows[b][c] = S_{c+1} (x) .. (x) S_{C-1} for c <= C - 2 (row C - 1 is left alone).
hipError_t words_scan(const WordTables& t, const float* S, int64_t B, int C, bool reverse, float* rows, float* last,
                      hipStream_t stream);
// Abar[b][c](u) = grad[b](u) + sum_v grad[b](u v) Q[b][c](v) for c <= C - 2; Q, Abar [B][C][W], rows C - 1 left alone
// both scans in one launch (two layers of workgroups): rows_forward as the forward scan's rows, rows_reverse as the reverse scan's
hipError_t words_scan_both(const WordTables& t, const float* S, int64_t B, int C, float* rows_forward, float* rows_reverse,
                           hipStream_t stream);
// zeroed: nullptr, or an array of n_zeroed floats that the kernel clears on the way
hipError_t words_adjoint(const WordTables& t, const float* grad, const float* Q, int64_t B, int C, float* Abar, float* zeroed,
                         int64_t n_zeroed, hipStream_t stream);

// Register-resident kernels for full truncations (kernels_trunc.hip)
bool trunc_forward_available(int d, int depth);
bool trunc_backward_available(int d, int depth);
int trunc_occupancy(int d, int depth, int backward);        // workgroups (of four wavefronts) resident per compute unit
int trunc_waves_per_row(int d, int depth, int backward);    // wavefronts per (path, chunk) row
// A path may be cut into C chunks of Lc segments (the last one shorter); every (path, chunk) pair is a row of its
// own in coeffs / grad_coeffs ([B * C, |W|]).  C = 1, Lc = P - 1 treats whole paths.
hipError_t trunc_forward(int d, int depth, const float* path, int64_t B, int64_t P, int64_t C, int64_t Lc, float* coeffs,
                         hipStream_t stream);
// Signatures over windows straight from the path: coeffs [B][K][|W|]; backward adds into gdx [B][P - 1][d] (zeroed by
// the caller; windows overlap) from coeffs / grad_coeffs [B][K][|W|].  Offered where trunc_forward / trunc_backward are.
hipError_t trunc_forward_windows(int d, int depth, const float* path, int64_t B, int64_t P, const WindowList& wl, float* coeffs,
                                 hipStream_t stream);
hipError_t trunc_backward_windows(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                                  int64_t P, const WindowList& wl, float* gdx, hipStream_t stream);
// tile: segments per LDS tile where a kernel offers a choice (d = 16: 8 or 16; 0 = the default)
// coeffs_last / grad_last (both or neither): [B][|W|] arrays that hold the rows of the last chunk of every path, while
// coeffs / grad_coeffs hold the other chunks' rows in [B][C][|W|] (the last slot of a path unused); nullptr: all rows
// are in coeffs / grad_coeffs.  resid: largest |coefficient| left in the signature reconstructed back to the start of
// every path (rows that begin at segment 0 report)
hipError_t trunc_backward(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs,
                          const float* coeffs_last, const float* grad_last, int64_t B, int64_t P, int64_t C, int64_t Lc,
                          float* gdx, float* resid /*[B], zeroed by the caller, or nullptr*/, int tile, hipStream_t stream);
const char* trunc_backward_kernel_name(int d, int depth);   // of the kernel trunc_backward launches

// d = 4: backward with one wavefront per row (a lane holds a word of length N - 3 and its four children); stores
// the gradient of the increments instead of accumulating, so the rows must tile every path exactly
bool trunc_backward_tails_available(int d, int depth);
hipError_t trunc_backward_tails(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                                int64_t P, int64_t C, int64_t Lc, float* gdx, float* grad_path /*C = 1: chain rule in the kernel*/,
                                hipStream_t stream);
// the same with the C = 2, 4 or 8 chunks of a path in one workgroup: chunk signatures, their products and the
// boundary adjoints stay in LDS; coeffs / grad_coeffs are [B, |W|]; writes the gradient with respect to the points
hipError_t trunc_backward_tails_fused(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs,
                                      int64_t B, int64_t P, int64_t C, int64_t Lc, float* grad_path, hipStream_t stream);
// forward with the C = 2 or 4 chunks of a path in one workgroup: chunk signatures multiplied in LDS; coeffs [B, |W|],
// 16-byte aligned
bool trunc_forward_tails_available(int d, int depth);
hipError_t trunc_forward_tails_fused(int d, int depth, const float* path, int64_t B, int64_t P, int64_t C, int64_t Lc,
                                     float* coeffs, hipStream_t stream);
hipError_t trunc_backward_tails_fused(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs,
                                      int64_t B, int64_t P, int64_t C, int64_t Lc, bool split, float* gdx, hipStream_t stream);

// Time chunks (kernels_chunk.hip): products of chunk signatures and adjoints at chunk boundaries, d a power of two
bool chunking_available(int d, int depth);
// forward: Q = terminal = nullptr, coeffs_out [B, |W|] receives the product of the C chunk signatures Sc [B, C, |W|];
// backward: coeffs_out = nullptr, Pfx [B, C, |W|] receives the signatures up to the end of every chunk (the last one
// is copied from terminal [B, |W|]) and Q [B, C, |W|] the signatures of the rest of the path after every chunk.
hipError_t chunk_scan(int d, int depth, const float* Sc, float* Pfx, float* Q, const float* terminal, float* coeffs_out,
                      const float* grad, float* Abar, int64_t B, int C, bool* adjoints_done, hipStream_t stream);
// (backward, small signatures: when grad [B, |W|] and Abar [B, C, |W|] are given the kernel also forms the boundary
// adjoints and *adjoints_done is set; otherwise call chunk_adjoint afterwards)
// Abar [B, C, |W|]: adjoint of the signature at the end of every chunk, from grad [B, |W|] and Q
// (skip_last: the last chunk's row of Abar, a copy of grad, is not written)
hipError_t chunk_adjoint(int d, int depth, const float* grad, const float* Q, float* Abar, int64_t B, int C, bool skip_last,
                         hipStream_t stream);

}  // namespace sig
