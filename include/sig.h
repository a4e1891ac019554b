/*
 * sig.h - C ABI of the MI355X (gfx950) path-signature library.
 *
 * What it computes: coefficients S_{0,T}(X, w) of the signature of batched
 * piecewise-linear paths for all words w of a prefix-closed word set W
 * (Section 3.1), and the gradient of a scalar loss with respect to the path
 * points given the gradient with respect to those coefficients (Section 4).
 *
 * Conventions
 *   - Letters are 0-based: {0, .., d-1} (Appendix A).
 *   - W never contains the empty word; its coefficient is the constant 1.
 *   - Canonical order of W: by word length, then lexicographic.  For a full
 *     depth-N truncation this is "cumulative level offset + base-d encoding"
 *     (Appendix A, word integer encoding), i.e. levels 1..N concatenated,
 *     each row-major.
 *   - A path is float32 [B, n_points, d], row-major, n_points = L + 1 >= 1.
 *   - coeffs / grad_coeffs are float32 [B, |W|] in canonical order; 16-byte aligned buffers get the fastest
 *     kernels (others fall back to kernels that read word by word; the long-path form with time chunks in the
 *     workspace returns SIG_EINVAL for them).
 *   - Every function returns 0 on success and a negative SIG_E* code on
 *     failure; nothing is printed, no exception or abort crosses the ABI.
 *   - "host" / "device" on a pointer says where the memory lives.  The library
 *     owns only sig_wordset objects (host memory).  All device memory is the
 *     caller's; the library never allocates or frees device memory.
 *   - sig_forward / sig_backward only enqueue work on the given HIP stream
 *     (hipStream_t passed as void*; NULL = the null stream) and return
 *     without synchronising.  Outputs are overwritten, never accumulated into.
 *   - The kernels are compiled for gfx950 only.
 */
#ifndef SIG_MI355X_H
#define SIG_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SIG_OK            0
#define SIG_EINVAL       (-1)  /* null pointer, d < 1, negative size, depth < 1, bad weights/cutoff, ... */
#define SIG_ELETTER      (-2)  /* a letter outside [0, d)                                                */
#define SIG_EEMPTYWORD   (-3)  /* the word list contains an empty word, or no word at all               */
#define SIG_ENOMEM       (-4)  /* host allocation failed                                                 */
#define SIG_EWORKSPACE   (-5)  /* workspace / table buffer missing or too small                          */
#define SIG_EHIP         (-6)  /* a HIP runtime call failed; see sig_last_hip_error()                    */
#define SIG_ETOOLARGE    (-7)  /* word set exceeds a format limit (see SIG_MAX_*)                        */
#define SIG_ENOTUPLOADED (-8)  /* sig_forward/sig_backward called before sig_wordset_upload              */
#define SIG_EUNSUPPORTED (-9)  /* word length above what the kernels handle (SIG_MAX_KERNEL_LEN)         */
#define SIG_ENOTREADY    (-11) /* sig_backward_static: the kernel for this set and batch is not loaded yet */

#define SIG_MAX_WORD_LEN    32          /* table format limit on |w|                                     */
#define SIG_MAX_KERNEL_LEN  12          /* longest word the GPU kernels handle                           */
#define SIG_MAX_WORDS       0x7fffffff  /* |W| < 2^31                                                    */

typedef struct sig_wordset sig_wordset;   /* opaque, host-owned */

/* ---- word-set construction (host, integer only; Section 3.1, Section 7, Appendix A) -------------------
 *
 * Each builder produces the canonical tables of a prefix-closed set:
 *   parent[w]      index of the word with the last letter removed, -1 if that is the empty word
 *   letter[w]      last letter of w
 *   level_start[n] index of the first word of length n, n = 1..max_len; level_start[0] = 0,
 *                  level_start[max_len + 1] = |W|
 * plus the launch plan the kernels use.  *out is set only on success and must be released
 * with sig_wordset_free.
 */

/* All words of length 1..depth over d letters (truncation pi_{<=N}, Section 2.1).  |W| = sum d^n. */
int sig_wordset_build_truncated(int d, int depth, sig_wordset** out);

/* All non-empty words with weighted degree <= cutoff (Definition 7.1).  weights: host, d doubles, each > 0.
 * The degree is accumulated left to right in double; a word is kept iff degree <= cutoff, no tolerance. */
int sig_wordset_build_anisotropic(int d, const double* weights, double cutoff, sig_wordset** out);

/* Arbitrary word list (word projection, Section 7.1) in CSR form: word k has letters
 * letters[offsets[k] .. offsets[k+1]).  Both arrays are host memory; offsets has n_words + 1
 * non-decreasing entries starting at 0.  Any order, duplicates allowed.  The list is closed under
 * prefixes; user_index[k] is the canonical index of word k in the closed set. */
int sig_wordset_build(int d, const int32_t* letters, const int64_t* offsets, int64_t n_words, sig_wordset** out);

/* Graph-induced set (Section 7.1): all words i_1..i_n, n <= depth, with (i_k, i_{k+1}) an edge for every k.
 * edges: host, n_edges pairs (from, to) of 0-based letters, duplicates allowed, any directed graph accepted.  Every
 * single letter is a word.  The set is prefix-closed by construction; user_index lists its words in canonical order. */
int sig_wordset_build_graph(int d, const int32_t* edges, int64_t n_edges, int depth, sig_wordset** out);

/* Sparse lead-lag set (Section 8) for a d-dimensional path after sig_leadlag_transform: alphabet of 2 d letters
 * (letter i = lag channel of coordinate i, letter d + i = its lead channel); all concatenations, of length <= depth,
 * of the generators (L_i), (l_i L_i), (L_i l_i).  That set is not prefix-closed: it is closed like any word list and
 * user_index gives the columns of the generated words (in order of the number of generators, then generator order). */
int sig_wordset_build_leadlag_sparse(int d, int depth, sig_wordset** out);

void sig_wordset_free(sig_wordset* ws);            /* NULL is allowed */

/* Accessors.  Returned host pointers stay valid until sig_wordset_free. */
int64_t        sig_wordset_size(const sig_wordset* ws);         /* |W|, empty word excluded; -1 if ws NULL */
int            sig_wordset_dim(const sig_wordset* ws);          /* d */
int            sig_wordset_max_len(const sig_wordset* ws);      /* longest word */
int64_t        sig_wordset_n_user(const sig_wordset* ws);       /* entries of user_index (0 unless built from a list) */
const int32_t* sig_wordset_parent(const sig_wordset* ws);       /* host [|W|] */
const int32_t* sig_wordset_letter(const sig_wordset* ws);       /* host [|W|] */
const int32_t* sig_wordset_level_start(const sig_wordset* ws);  /* host [max_len + 2] */
const int64_t* sig_wordset_user_index(const sig_wordset* ws);   /* host [n_user] or NULL */
/* Sets other than full truncations that are closed under suffixes as well as prefixes (every anisotropic set of
 * Definition 7.1; word lists that happen to be): the product of Section 2.1 restricted to such a set needs no word
 * outside it, which is what the checkpointed calls below need.  sig_wordset_suffix_closed: 1 / 0 (-1 if ws NULL; 0 for
 * full truncations, which have product kernels of their own).  sig_wordset_tail_table: host tables or NULL; for a
 * word w of length n >= 2 and m = 1 .. n - 1, the index of w without its first m letters is
 * tail_tab[tail_off[n] + (m - 1) * (level_start[n + 1] - level_start[n]) + (w - level_start[n])]; tail_off has
 * max_len + 2 entries. */
int            sig_wordset_suffix_closed(const sig_wordset* ws);
const int32_t* sig_wordset_tail_table(const sig_wordset* ws, const int32_t** tail_off);
/* The terms (w, m) of the product (a (x) b)(w) = a(w) + b(w) + sum_m a(w_1..w_m) b(w_m+1..w_n) as the kernels of the
 * checkpointed calls read them (suffix-closed sets of up to 65,535 words; returns -1 otherwise), host arrays:
 * prod_pairs, laid out like the tail table, entry (m, w) = prefix | suffix << 16; adj_pairs / adj_key, the same terms
 * sorted by their prefix u = w_1..w_m: adj_pairs = w | suffix << 16, adj_key = u, *n_adj entries, a multiple of 256
 * (padding entries carry the key |W|).  Returns the number of entries of prod_pairs. */
int64_t        sig_wordset_term_tables(const sig_wordset* ws, const uint32_t** prod_pairs, const uint32_t** adj_pairs,
                                       const uint32_t** adj_key, int64_t* n_adj);

/* Launch-shape knobs of a word set.  They are filled once, when the set is built, from the environment variables in
 * brackets, and changed afterwards only through sig_wordset_set_option; sig_forward / sig_backward never read the
 * environment.  The launcher's own choice is the default; the knobs exist for tests and tuning scans.
 *   "no_jit"        [SIG_NO_JIT]         1: table-driven kernels instead of run-time specialised ones
 *   "jit_waves"     [SIG_JIT_WAVES]      wavefronts the balanced plan of the specialised kernels aims at (0: 2,048)
 *   "chunks"        [SIG_CHUNKS]         time chunks with the chunk arrays in the workspace (0: launcher decides)
 *   "fwd_tails"     [SIG_FWD_TAILS]      d = 4 forward with the chunks of a path in one workgroup: -1 auto, 0 off, 2, 4
 *   "bwd_tails"     [SIG_BWD_TAILS]      d = 4 backward: -1 auto, 0 off, 1 one wavefront per row, 2 / 4 / 8 fused chunks
 *   "lanes"         [SIG_LANES]          word-per-lane kernels for full truncations: -1 auto, 0 off, 1 wherever defined
 *   "lanes_levels"  [SIG_LANES_LEVELS]   levels below the lane's word: 0 auto, 1, 2
 *   "logsig_gather" [SIG_LOGSIG_GATHER]  1: two-kernel form of sig_logsig_backward
 *   "jit_wg_waves"  [SIG_JIT_WG_WAVES]   wavefronts per workgroup of the specialised kernels, 1..4 (default 4)
 *   "bwd_tile"      [SIG_BWD_TILE]       LDS tile of the backward kernels, 0 = launcher's rule.  d = 8: 4, 8 or 16 segments;
 *                                        d = 16: 8, 12 or 16 segments, or 4 = 16 segments with the gradient sources
 *                                        summed every 4 (the form that fits two workgroups on a compute unit)
 *   "ckpt_chunks"   [SIG_CKPT_CHUNKS]    time chunks of the checkpointed calls: 0 launcher's rule, 1 off, 2..16 forced
 *   "jit_fwd_tile"  [SIG_JIT_FWD_TILE]   segments per LDS tile of the specialised forward kernels: 0 default, 1..32
 * Workspace sizes depend on the knobs: query them again after a change.  Returns SIG_EINVAL for an unknown name.
 * Not to be called while another thread runs sig_forward / sig_backward on the same word set. */
int sig_wordset_set_option(sig_wordset* ws, const char* name, int value);
int sig_wordset_get_option(const sig_wordset* ws, const char* name, int* value);

/* Multiply-adds one path needs per segment when Horner intermediates are shared between words with a
 * common prefix: sum over words u of (1 + height of the sub-tree under u).  This is the work unit the
 * benchmark prices against the FP32 vector peak (Algorithm 1 evaluated once per (prefix, target length)). */
int64_t sig_wordset_min_fma_per_step(const sig_wordset* ws);
/* Multiply-adds per path and segment that the forward / backward kernels actually issue for this set
 * (includes recomputation of shared ancestors in each work unit). */
int64_t sig_wordset_kernel_fma_per_step(const sig_wordset* ws, int backward);

/* Launch-plan introspection (host).  The word tree is split into work units; each unit has a program
 * (pre-order walk, one 32-bit op per word: bits 0..11 last letter, 12..15 word length, 16..19 height of
 * the word's sub-tree inside the unit, 20..21 kind 0 = leaf, 1 = enter, 2 = leave [backward plans only])
 * and a slot table (canonical word index per leaf/enter op in program order; a negative value ~index marks
 * a shared ancestor this unit only recomputes).  Several variants exist per direction, coarse to fine.
 * units: int32 [n_units][4] = {first op, op count, first slot, slot count}.  Any output pointer may be
 * NULL.  Returns SIG_EINVAL for a bad variant. */
int sig_wordset_plan_count(const sig_wordset* ws, int backward);
int sig_wordset_plan_get(const sig_wordset* ws, int backward, int variant, const int32_t** units, int64_t* n_units,
                         const uint32_t** ops, int64_t* n_ops, const int32_t** slot_word, int64_t* n_slots,
                         int64_t* fma_per_step);

/* Run-time specialisation.  For word sets without a precompiled register-resident kernel, sig_forward and
 * sig_backward print the work units as straight-line HIP source (one multiply-add per (word, target length)
 * pair) and compile it with hiprtc for gfx950 on first use; the compiled kernel is cached in ws.  The first call
 * for a word set therefore takes seconds.  sig_wordset_jit_prepare does that compilation ahead of time for the
 * plan variant a batch of B paths would use (host only, no device needed); it returns SIG_OK, SIG_EUNSUPPORTED if
 * this word set is not run through specialised kernels, or SIG_EJIT if hiprtc failed (sig_forward / sig_backward
 * then fall back to the table-driven kernels).  The option "no_jit" disables it.
 * Full truncations (any d <= 64) without a precompiled kernel are the exception to "grows with the word set": they
 * run one fixed kernel source with a word per lane, compiled for the shape (d, depth) in under a second per
 * direction (Section 3.1, eq. (3), with the prefixes shared between words); the option "lanes" = 0 sends them through
 * the straight-line form as well, = 1 takes the word-per-lane form even where a path has only a few words of
 * length depth - 2.  sig_wordset_jit_prepare and sig_wordset_jit_source cover whichever form the batch would use.
 * With the environment variable SIG_JIT_CACHE naming an existing directory (read when a kernel is compiled), code
 * objects are kept there (named by a hash of their source, the compiler version and the compile options; each file
 * carries its length and a checksum) and later processes load them instead of compiling; a file that fails its
 * checks or does not load is removed and replaced.
 * Threads: calls on different word-set objects may run concurrently; a compilation holds only its own kernel's lock.
 * A word-set object serves the device it was uploaded on. */
#define SIG_EJIT (-10)
int sig_wordset_jit_prepare(sig_wordset* ws, int backward, int64_t B);
/* The plan the specialised kernel for a batch of B paths is generated from, in the format of sig_wordset_plan_get.
 * Here the words in depth-first order are cut into consecutive runs of nearly equal cost, one per wavefront, as
 * many as the batch needs to occupy the chip; a unit is one run plus the ancestors of its first word.  Pointers
 * stay valid until sig_wordset_free.  Host only. */
int sig_wordset_jit_plan_get(sig_wordset* ws, int backward, int64_t B, const int32_t** units, int64_t* n_units,
                             const uint32_t** ops, int64_t* n_ops, const int32_t** slot_word, int64_t* n_slots,
                             int64_t* fma_per_step);
/* Copies the generated source (NUL-terminated, truncated to n bytes) and returns its full length, 0 if none. */
size_t sig_wordset_jit_source(sig_wordset* ws, int backward, int64_t B, char* buf, size_t n);
/* The check every run-time compiled kernel passes before it may be launched, as a function of what the loaded code
 * object declares (host only; 1 = may be launched).  A kernel of `waves` wavefronts per workgroup is refused when
 * waves * 64 exceeds max_threads_per_block, when its static LDS exceeds the 64 KB a kernel may use without opting in
 * (the shape of a dispatch that the runtime rejected: 8 wavefronts with 112 KB of static LDS), or when its registers
 * do not fit the wavefronts of a workgroup that share a SIMD (512 per lane).  A refused kernel is never dispatched; the
 * table-driven kernels run instead. */
int sig_jit_launch_shape_ok(int waves, int max_threads_per_block, int static_lds_bytes, int registers);

/* ---- device tables ------------------------------------------------------------------------------------
 * The kernels read the launch plan from device memory the caller provides.  Allocate
 * sig_wordset_device_bytes(ws) bytes (256-byte aligned), then call sig_wordset_upload once; the buffer
 * must outlive every sig_forward / sig_backward call that uses ws.  The copy is enqueued on `stream`
 * from host memory owned by ws. */
size_t sig_wordset_device_bytes(const sig_wordset* ws);
int    sig_wordset_upload(sig_wordset* ws, void* dev_buf /*device*/, size_t dev_bytes, void* stream);

/* ---- forward (Section 3: Chen's relation per segment, Algorithm 1 / eq. 3 per word) -------------------
 * path   device float32 [B, n_points, d]
 * coeffs device float32 [B, |W|]            fully overwritten
 * workspace: device, sig_forward_workspace_bytes bytes (may be 0 -> NULL allowed), 256-byte aligned,
 *            contents undefined before and after.
 * Full truncations with few paths are cut into time chunks that run side by side and are multiplied together
 * afterwards (Chen's relation, eq. 2, is associative); sig_backward does the same where four or more chunks fit
 * (or on request, option "chunks") and recomputes the chunk signatures from the path.  Word sets closed under suffixes (sig_wordset_suffix_closed) that run through the
 * run-time specialised kernels take the chunks of the checkpointed calls below in sig_forward as well, with the
 * chunk signatures in the workspace; sig_backward recomputes them and does the same from four chunks on (few long
 * paths), where that still beats walking whole paths.
 * n_points == 1 gives all-zero coeffs (S_{0,0} = 1 has no non-empty-word part).  B == 0 is a no-op. */
size_t sig_forward_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points);
int    sig_forward(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, float* coeffs,
                   void* workspace, size_t workspace_bytes, void* stream);

/* ---- backward (Section 4: Proposition 4.1 gradient, Proposition 4.6 reconstruction of S_{0,t_j} by
 *      exp(-dX_j), chain rule from increments to points) ------------------------------------------------
 * coeffs      device float32 [B, |W|]  the terminal signature sig_forward produced for the same path
 * grad_coeffs device float32 [B, |W|]  dLoss/dS_{0,T}(w); use 0 for words the loss does not depend on
 * grad_path   device float32 [B, n_points, d]  fully overwritten with dLoss/dX
 * Only the terminal signature is needed; no per-step state is stored (Section 4.2).
 * Partial gradients of different work units are combined with floating-point atomics, so the last bits
 * of grad_path may differ from run to run. */
size_t sig_backward_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points);
int    sig_backward(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs,
                    int64_t B, int64_t n_points, float* grad_path, void* workspace, size_t workspace_bytes,
                    void* stream);

/* sig_backward with a check of the reconstruction it rests on (Lemma 4.5, Proposition 4.6): stepping the terminal
 * signature back through all segments must end at the signature of the empty path, whose coefficients of non-empty
 * words are zero.  residual: device float32 [B], receives per path the largest absolute value left in the
 * reconstructed coefficients (words shorter than the depth: the longest words are never reconstructed).  Offered for
 * the full truncations with a precompiled kernel (SIG_EUNSUPPORTED otherwise); runs the kernel that walks whole paths,
 * so it measures the drift over all L segments.  Workspace as for sig_backward. */
int    sig_backward_residual(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs,
                             int64_t B, int64_t n_points, float* grad_path, float* residual /*device [B]*/,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ---- forward and backward with time chunks kept between the two calls --------------------------------------------
 * Chen's relation (eq. 2) lets a path be cut into C consecutive chunks whose signatures multiply to the signature of
 * the path.  sig_forward_checkpointed computes the chunk signatures side by side, leaves them in `checkpoint` (device,
 * [B, C, |W|] float32, 256-byte aligned, sig_checkpoint_bytes bytes, the caller's to keep until the backward call)
 * and writes their product to coeffs.  sig_backward_checkpointed then walks the C chunks of every path side by side:
 * the signature at the end of chunk c is the product of the first c chunk signatures, the adjoint there is
 * Abar_c(u) = sum_v grad_coeffs(u v) Q_c(v) with Q_c the product of the chunk signatures after c (Proposition 4.1
 * with the right factor taken at a chunk boundary), and inside a chunk the recursion is that of sig_backward
 * (Proposition 4.6).  Nothing is recomputed; the price is C times the memory of coeffs between the two calls, where
 * sig_forward / sig_backward keep the terminal signature alone (Section 4.2).  The library picks C for the batch
 * (2 .. 16): for full truncations whose backward kernel would otherwise leave SIMDs with a single wavefront (few
 * paths with many segments), and for suffix-closed sets (sig_wordset_suffix_closed) of up to 13,653 words that run
 * through the run-time specialised kernels, which gain from more rows (up to eight chunks: at most 2,048 rows,
 * chunks of at least 256 segments, 128 for batches that stay at 512 rows or below).  Where it sees no gain sig_checkpoint_bytes is 0, `checkpoint` is not touched and
 * the two calls are sig_forward / sig_backward; the same holds when a specialised kernel cannot be compiled (then
 * `checkpoint` is left alone by both calls).  Results agree with sig_forward / sig_backward to rounding. */
size_t sig_checkpoint_bytes(const sig_wordset* ws, int64_t B, int64_t n_points);
/* The number of time chunks C the two calls take for this batch (1: none, the calls are sig_forward / sig_backward).
 * For a suffix-closed set the specialised kernels of the checkpointed calls run B * C rows: compile them ahead of time
 * with sig_wordset_jit_prepare(ws, backward, B * C). */
int64_t sig_checkpoint_chunks(const sig_wordset* ws, int64_t B, int64_t n_points);
size_t sig_forward_checkpointed_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points);
size_t sig_backward_checkpointed_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points);
int    sig_forward_checkpointed(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, float* coeffs,
                                void* checkpoint, size_t checkpoint_bytes, void* workspace, size_t workspace_bytes,
                                void* stream);
int    sig_backward_checkpointed(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs,
                                 const void* checkpoint, size_t checkpoint_bytes, int64_t B, int64_t n_points,
                                 float* grad_path, void* workspace, size_t workspace_bytes, void* stream);

/* The same computation for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): no workspace argument; the buffers sig_backward takes from its workspace
 * (gradient with respect to the increments, transposed increments, chunk arrays) live in a static device array of
 * SIG_STATIC_SCRATCH_BYTES that each GPU the library runs on holds until the process ends.  The call allocates nothing
 * and frees nothing; it only enqueues kernels on `stream` (what must start at zero is cleared by a kernel first).
 * Errors beyond those of sig_backward: SIG_ETOOLARGE when sig_backward_workspace_bytes(ws, B, n_points) exceeds
 * SIG_STATIC_SCRATCH_BYTES; SIG_ENOTREADY when the word set runs through a run-time compiled kernel that this process
 * has not loaded yet (loading a code object allocates): one sig_backward call of the same batch size loads it.
 * All calls on one GPU share that GPU's array: calls that overlap in time on the same device (different streams or
 * host threads) race; calls on one stream are ordered and safe. */
#define SIG_STATIC_SCRATCH_BYTES (32u << 20)
int    sig_backward_static(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs,
                           int64_t B, int64_t n_points, float* grad_path, void* stream);

/* ---- log-signature (Section 3.3) -----------------------------------------------------------------------------
 * Coordinates: for every Lyndon word w of length <= depth, the coefficient of w in the tensor logarithm of the
 * signature (the Lyndon-word coordinates the paper takes from its reference on efficient Lie bases).  Only the
 * coefficients of the factors of Lyndon words are needed: sig_wordset_build_logsig builds the set "every word shorter
 * than depth + the Lyndon words of length depth" (the full truncation instead for the (d, depth) pairs that have
 * a kernel of their own for it: faster, and a superset); user_index lists the columns of the Lyndon words (by length, then
 * lexicographic), sig_wordset_n_lyndon their number.  Pipeline: sig_forward on that set, then sig_logsig_forward
 * (coeffs [B, |W|] -> logsig [B, n_lyndon]); backward: sig_logsig_backward (grad_logsig -> grad_coeffs [B, |W|],
 * overwritten), then sig_backward.  All pointers device, float32; the word set must be uploaded. */
int     sig_wordset_build_logsig(int d, int depth, sig_wordset** out);
int64_t sig_wordset_n_lyndon(const sig_wordset* ws);
int     sig_logsig_forward(const sig_wordset* ws, const float* coeffs, int64_t B, float* logsig, void* stream);
size_t  sig_logsig_backward_workspace_bytes(const sig_wordset* ws, int64_t B);
int     sig_logsig_backward(const sig_wordset* ws, const float* coeffs, const float* grad_logsig, int64_t B, float* grad_coeffs,
                            void* workspace /*device*/, size_t workspace_bytes, void* stream);

/* ---- signatures over windows (Section 5) -------------------------------------------------------------------
 * windows: device int64 [K][2], point indices (l_k, r_k) with 0 <= l_k <= r_k < n_points; window k is the path
 *          restricted to the points l_k .. r_k (segments l_k .. r_k - 1; l_k == r_k gives the zero signature).
 *          Indices outside the path are clamped.  max_window_len (host) >= max_k (r_k - l_k): the library cannot
 *          read the device array, a longer window is cut after max_window_len segments.
 * coeffs / grad_coeffs: device float32 [B, K, |W|];  grad_path: device float32 [B, n_points, d], overwritten with
 *          the sum over the windows (floating-point atomics).
 * All windows of all paths advance side by side in one launch.  Full truncations with a precompiled kernel (d, depth)
 * in {(4, 6), (8, 5), (16, 4)} read every window straight from the path as a row of its own (no copy, a short window
 * ends early, the gradients of overlapping windows are added up in the increment-gradient array), and so do the
 * word-per-lane kernels of the other full truncations; word sets that run through the straight-line specialised
 * kernels take their rows' increments straight from the path as well (a short window is padded with zero increments)
 * and add the rows' gradients into grad_path.  Only the table-driven fallback gathers every (path, window) pair into a
 * path of max_window_len + 1 points (shorter windows padded with their last point) and scatters the gradient back.
 * Workspace sizes from the two functions below (256-byte aligned). */
size_t sig_forward_windows_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points, int64_t K, int64_t max_window_len);
size_t sig_backward_windows_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points, int64_t K, int64_t max_window_len);
int sig_forward_windows(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, const int64_t* windows, int64_t K,
                        int64_t max_window_len, float* coeffs, void* workspace, size_t workspace_bytes, void* stream);
int sig_backward_windows(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                         int64_t n_points, const int64_t* windows, int64_t K, int64_t max_window_len, float* grad_path,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ---- lead-lag transform (Section 8, Definition of the lead-lag path) ------------------------------------------
 * path device float32 [B, n_points, d] -> out device float32 [B, 2 n_points - 1, 2 d]:
 * out[2k] = (X_k, X_k), out[2k+1] = (X_k, X_{k+1}); channels 0..d-1 lag, d..2d-1 lead.  sig_leadlag_backward maps
 * grad_out [B, 2 n_points - 1, 2 d] to grad_path [B, n_points, d] (overwritten).  Both only enqueue on `stream`. */
int sig_leadlag_transform(const float* path, int64_t B, int64_t n_points, int d, float* out, void* stream);
int sig_leadlag_backward(const float* grad_out, int64_t B, int64_t n_points, int d, float* grad_path, void* stream);

/* ---- kernel timer ----------------------------------------------------------------------------------------
 * For benchmarks: while enabled, sig_forward / sig_backward record two HIP event pairs on the caller's stream:
 * one around their main kernel (the hot loop over segments) and one around everything the call enqueues (with
 * the small fill / transpose / chunk-product / chain-rule kernels).  sig_profile_read synchronises with the
 * recorded events and returns the number of calls recorded since sig_profile_enable(1) and the sum of the
 * durations in milliseconds for `which` = 0 forward main kernel, 1 backward main kernel, 2 whole forward call,
 * 3 whole backward call.  sig_profile_enable(0) switches recording off, (1) switches all four channels on, and
 * (2 << which, or several of these or-ed) only the named ones: every recorded event costs a few microseconds on
 * the stream, so a timed region that needs one kernel's duration enables that channel alone.  At most
 * SIG_PROFILE_MAX_LAUNCHES calls per channel are kept; later ones are not recorded.  Not thread-safe; events are
 * created on first use (no device memory is allocated). */
#define SIG_PROFILE_MAX_LAUNCHES 4096
int sig_profile_enable(int on);
int sig_profile_read(int which, int64_t* n_launches, double* total_ms);

/* Vector-ALU rate probe for benchmarks: enqueues a register-only kernel of `blocks` workgroups of 256 threads in
 * which every thread performs iters * 16 dependent-chain-free fmaf operations (2 * 16 * iters * 256 * blocks
 * floating-point operations in all) and stores one float; out: device, blocks * 256 floats.  The caller times it. */
int sig_probe_fma(void* out /*device*/, size_t out_bytes, int blocks, int iters, void* stream);

/* Issue-rate probes for benchmarks: register-only loops of `blocks` workgroups of 256 threads (one wavefront per SIMD of
 * a compute unit per workgroup); per iteration a wavefront issues, by `mode`,
 *   0: 64 multiply-adds whose operands are all vector registers      1: 64 multiply-adds with a scalar-register multiplier
 *   2: 8 matrix instructions 16x16x4 (fp32)                            3: the 64 multiply-adds of 0 interleaved with the 8 of 2
 *   4: 64 multiply-adds whose three source registers share a register bank (register number mod 4)
 *   5: the same with the three source registers in three different banks
 *   6: accumulator and multiplier in one bank, the addend in another      7: multiplier and addend in one bank, the accumulator in another
 *      (4 .. 7 name their registers in the instruction)
 * out: device, blocks * 256 floats.  The caller times the launch; with 256 blocks a SIMD holds one wavefront, with 512 two. */
int sig_probe_issue(void* out /*device*/, size_t out_bytes, int blocks, int iters, int mode, void* stream);

/* ---- diagnostics ------------------------------------------------------------------------------------- */
const char* sig_strerror(int code);
int         sig_last_hip_error(void);          /* hipError_t of the last SIG_EHIP on this thread, else 0 */
const char* sig_version(void);
/* Name of the kernel family sig_forward / sig_backward will launch for this set ("generic", "trunc<d,N>", ...);
 * lets a benchmark say which kernel its numbers belong to. */
const char* sig_wordset_kernel_name(const sig_wordset* ws, int backward);
/* The same for a given batch: which main kernel sig_forward / sig_backward launch for B paths of n_points points. */
const char* sig_kernel_name(const sig_wordset* ws, int backward, int64_t B, int64_t n_points);

#ifdef __cplusplus
}
#endif
#endif /* SIG_MI355X_H */
