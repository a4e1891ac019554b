// Host-side word set: canonical tables of a prefix-closed set (Section 3.1, Appendix A) and the
// launch plans the kernels read.  Integer work only.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

namespace sig {

// One instruction of a work unit's program.  A work unit is a connected piece of the word tree
// that contains the root side of every word in it: a chain of ancestors (recomputed by every unit
// that needs them) followed by complete sub-trees.  The program is the pre-order walk of that piece.
//   bits  0..11  last letter of the word
//   bits 12..15  word length k (1..15)
//   bits 16..19  h = height of the word's sub-tree inside this unit (number of longer target
//                lengths whose Horner intermediate passes through this word)
//   bits 20..21  kind: 0 = LEAF (h == 0), 1 = ENTER (h >= 1), 2 = LEAVE (closes the matching ENTER;
//                emitted for backward programs only)
enum : uint32_t { OP_LEAF = 0, OP_ENTER = 1, OP_LEAVE = 2 };
inline uint32_t op_pack(uint32_t letter, uint32_t level, uint32_t h, uint32_t kind) {
    return letter | (level << 12) | (h << 16) | (kind << 20);
}

struct JitKernel;          // jit.hpp

struct UnitDesc {          // device-visible, 16 bytes
    int32_t op_off;        // first op in Plan::ops
    int32_t n_ops;
    int32_t slot_off;      // first entry in Plan::slot_word
    int32_t n_slots;       // words held by the unit (one LDS row each)
};

struct Plan {
    std::vector<UnitDesc> units;
    std::vector<uint32_t> ops;
    // Canonical word index of every slot, in slot order (= order of LEAF/ENTER ops).  A unit that
    // carries a word only as a recomputed ancestor stores ~index (negative): it reads the word's
    // coefficient but neither writes it nor seeds its adjoint.
    std::vector<int32_t> slot_word;
    int32_t max_slots = 0;         // largest n_slots
    int64_t fma_per_step = 0;      // multiply-adds per path and segment issued over all units (forward count)
    int64_t pairs_nonleaf = 0;     // (word, target) pairs with target length > word length, over all units
    int64_t leaves = 0;            // LEAF ops over all units
};

struct WordSet {
    int d = 0;
    int max_len = 0;
    int kind = 0;                  // 0 truncated, 1 anisotropic, 2 list
    int depth = 0;                 // truncated only
    std::vector<int32_t> parent, letter, level_start;
    std::vector<int64_t> user_index;
    // tree
    std::vector<int32_t> child_off;    // [|W|+2]: children of word w are child_list[child_off[w+1] .. child_off[w+2]);
                                       // entry 0 describes the empty word (the roots = words of length 1)
    std::vector<int32_t> child_list;
    std::vector<uint8_t> height;       // height of the sub-tree under w (0 for a leaf)
    std::vector<uint8_t> length;
    int64_t min_fma = 0;               // sum over words of (1 + height)
    // Plan variants, coarse to fine (fewer, larger units first).  plans[0]: forward programs,
    // plans[1]: backward programs (with LEAVE ops, smaller units because two values per word are held).
    std::vector<Plan> plans[2];
    // device image: all plans back to back, every array 256-byte aligned
    struct PlanOffsets { size_t units, ops, slots; };
    std::vector<PlanOffsets> offsets[2];
    std::vector<unsigned char> image;
    // log-signature (sets built by build_logsig only): for every Lyndon word of length <= depth, its length and the
    // canonical indices of all its contiguous sub-words w[i:j], 0 <= i < j <= n, at lyn_sub[k * lyn_stride + i * (depth + 1) + j]
    int64_t n_lyndon = 0;
    int lyn_stride = 0;
    std::vector<int32_t> lyn_len, lyn_sub;
    // inverse of lyn_sub for the backward pass: word u is the factor w_k[i:j] for the entries
    // lyn_inv[lyn_inv_off[u] .. lyn_inv_off[u + 1]), each k * lyn_pairs + pair(i, j), pair(i, j) counting the pairs
    // i < j <= depth in the order i = 0.., j = i + 1..
    int lyn_pairs = 0;
    std::vector<int32_t> lyn_inv_off, lyn_inv;
    size_t lyn_len_off = 0, lyn_sub_off = 0, lyn_inv_off_off = 0, lyn_inv_ent_off = 0;    // offsets in the device image
    // Sets closed under suffixes as well (every anisotropic set; word lists that happen to be): the tensor product of
    // two elements restricted to the set needs nothing outside it, (a (x) b)(w) = sum_k a(w_1..k) b(w_k+1..n), so the
    // segments of a path can be cut into time chunks whose signatures are multiplied afterwards (Chen's relation).
    // tail_tab: for every length n >= 2 and m = 1..n-1, the index of each word of length n without its first m
    // letters, at tail_tab[tail_off[n] + (m - 1) * (words of length n) + (w - level_start[n])].
    bool suffix_closed = false;
    std::vector<int32_t> tail_tab;
    std::vector<int32_t> tail_off;     // [max_len + 2]
    // the terms of the product in the two orders the kernels read, two 16-bit word indices per entry (see wordset.cpp)
    bool pair_tables = false;
    std::vector<uint32_t> prod_pairs, adj_pairs, adj_key;
    std::vector<int32_t> adj_off;      // [|W| + 1] (host only)
    size_t dev_prod_off = 0, dev_adj_key_off = 0, dev_adj_pairs_off = 0;    // offsets in the device image (pair_tables only)
    void* dev = nullptr;
    int dev_id = -1;                   // device the image was uploaded to (a word-set object serves one device)
    // Launch-shape knobs.  Filled once when the set is built (from the SIG_* environment variables of that moment) and
    // changed afterwards only through sig_wordset_set_option; no entry point reads the environment per call.
    struct Options {
        int no_jit = 0;                // 1: table-driven kernels instead of run-time specialised ones
        int jit_waves = 0;             // wavefronts the balanced plan aims at (0: two per SIMD)
        int chunks = 0;                // time chunks with the chunk arrays in the workspace (0: the launcher decides)
        int fwd_tails = -1;            // d = 4 forward, chunks of a path in one workgroup: -1 auto, 0 off, 2 / 4 forced
        int bwd_tails = -1;            // d = 4 backward: -1 auto, 0 off, 1 one wavefront per row, 2 / 4 / 8 fused chunks
        int lanes = -1;                // word-per-lane kernels for full truncations: -1 auto, 0 off, 1 whenever defined
        int lanes_levels = 0;          // levels below the lane's word: 0 auto, 1, 2
        int logsig_gather = 0;         // 1: two-kernel form of the log-signature adjoint
        int ckpt_chunks = 0;           // time chunks of the checkpointed forward / backward: 0 launcher's rule, 1 off, 2..4
        int bwd_tile = 0;              // LDS tile shape of the d = 8 (4, 8) and d = 16 (4, 8, 12, 16) backward kernels; 0: launcher's rule
        int jit_fwd_tile = 0;          // segments per LDS tile of the specialised forward kernels: 0 default, 1..32
        int jit_wg_waves = 4;          // wavefronts (work units) per workgroup of the run-time specialised kernels, 1..4;
                                       // 8 is accepted for inspecting the generated code on the host only: jit_load
                                       // refuses code objects whose registers do not fit two wavefronts per SIMD
    } opt;
    bool kernels_supported = true;     // false when max_len exceeds what the kernels handle
    // run-time specialised kernels with the balanced plan each was generated from, per direction, keyed by the
    // number of work units asked for; built on first use
    struct JitEntry {
        int64_t n_units = 0;
        int wg_waves = 0;              // wavefronts per workgroup the kernel is generated for
        int tile = 0;                  // segments per LDS tile the kernel is generated for
        Plan plan;
        JitKernel* kernel = nullptr;
    };
    std::vector<JitEntry*> jit[2];
    // full truncations: kernels with lanes = words, per direction and levels per lane (jit_lanes.cpp); built on
    // first use
    JitKernel* lanes[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
    WordSet() = default;
    WordSet(const WordSet&) = delete;
    WordSet& operator=(const WordSet&) = delete;
    ~WordSet();                        // defined in jit.cpp (releases the compiled kernels)

    int64_t size() const { return (int64_t)parent.size(); }
};

int build_truncated(int d, int depth, WordSet** out);
int build_anisotropic(int d, const double* weights, double cutoff, WordSet** out);
int build_list(int d, const int32_t* letters, const int64_t* offsets, int64_t n_words, WordSet** out);
int build_graph(int d, const int32_t* edges, int64_t n_edges, int depth, WordSet** out);
int build_leadlag_sparse(int d, int depth, WordSet** out);
// Word set for the log-signature of depth `depth` in the Lyndon-word coordinates: every word shorter than depth and
// the Lyndon words of length depth; user_index lists the Lyndon words of all lengths (by length, then lexicographic).
int build_logsig(int d, int depth, WordSet** out);

// Splits the word tree into work units of at most max_slots words and about target_cost multiply-adds.
void build_plan(const WordSet& ws, int max_slots, int64_t target_cost, bool with_leave, Plan& plan);


// Balanced split for the run-time specialised kernels: the words in depth-first order are cut into at most
// n_units consecutive runs of (nearly) equal cost; a unit is one run plus the ancestors of its first word
// (recomputed, owned by an earlier unit).  Cost of a word = cost_word + cost_pair * (height of its sub-tree inside
// the unit).  No unit holds more than max_slots words.
void build_plan_balanced(const WordSet& ws, int64_t n_units, int max_slots, bool with_leave, int cost_word, int cost_pair,
                         Plan& plan);

}  // namespace sig
