// Device-visible model description shared by the kernels and the host glue.
// gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace amusd {

constexpr int kRows = 16;          // rows of a pass = one matrix-core tile
constexpr int kWaves = 8;          // waves per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kMaxTilesPerRound = 8;

constexpr int kSplitWaysMax = 2;   // K ranges a stage's tiles can be split into across workgroups
constexpr int kSplitTickets = 512; // pairs of workgroups that can share tiles in one stage (compute units / 2 at most)

constexpr int kMaxSegs = kRows;    // a pass serves at most one sequence per row

// One sequence's share of a pass: rows row0 .. row0+k-1 of the tile are its
// tokens for positions L .. L+k-1, checked against its own cache (slot).
struct PassSeg {
    int L;        // cache length of the sequence before the pass (ctx_len)
    int k;        // rows of this sequence
    int row0;     // first tile row
    int p_ctx;    // model's greedy token for position L
    int slot;     // which key-value cache
    int unit0;    // first attention work unit of the sequence
    int nchunks;  // attention chunks covering positions 0 .. L+k-1
    int pad;
};

// Per-pass values.  They travel as kernel arguments (no device round trip
// before the first weight load can be addressed).
struct PassArgs {
    int k;              // rows of the pass, all sequences together
    int n_seg;          // sequences in the pass
    int force_accept;   // 1: prefill, every row is kept
    int keep_logits;    // 1: store fp32 logits
    // The first sequence's values once more, next to k: a pass of ONE sequence (the usual case) then needs nothing
    // from the per-row and per-segment tables below, which a lane can only reach through dependent loads of the
    // argument memory (a memory round trip each, before the kernel's first useful address is known).
    int L0;             // seg[0].L
    int slot0;          // seg[0].slot
    int nchunks0;       // seg[0].nchunks
    int units;          // attention work units of the pass, all sequences together
    int tokens[kRows];  // input token of each row
    int row_pos[kRows]; // position of each row in its sequence
    int row_seg[kRows]; // segment of each row
    PassSeg seg[kMaxSegs];
};

struct PassResult {
    int accept_len[kMaxSegs];   // per segment
    int next_token[kMaxSegs];
    int greedy[kRows];          // per row
};

struct DevLayer {
    const uint4* wqkv;   // fragment-ordered [ (Hq+2Hkv)*hd/16 tiles ][ d/KB ][64 lanes] x 16 B
    const uint4* wo;     // [d/16][qdim/KB][64]
    const uint4* wgu;    // [2F/16][d/KB][64]   tile t: rows 0-7 gate features 8t.., rows 8-15 up features 8t..
    const uint4* wd;     // [d/16][F/KB][64]
    const float* g_attn; // [d]
    const float* g_mlp;  // [d]
    void* kcache;        // [slot][Hkv][ctx_pad/16][hd/4/EPL][64 lanes][EPL] elements (operand order of the score product)
    void* vcache;        // [slot][Hkv][ctx_pad/BK][hd/16][64 lanes][EPL] elements (matrix-core operand order)
};

struct DevModel {
    int n_layers, d, Hq, Hkv, hd, F, V, G;
    int qdim, kvdim, nqkv;
    int max_ctx, ctx_pad;
    int n_slots;          // key-value caches (sequences the model can hold)
    int dtype;
    int chunk;            // keys per attention work unit: (8/G) runs x bpw blocks x keys-per-block
    int bpw;              // key blocks a wave walks in one attention work unit
    int max_chunks;
    int lm_wgs;           // workgroups that produce arg-max partials
    int split_down;       // tiles per pair of workgroups that share their K range in the down projection (0: no sharing)
    float eps, att_scale;
    const DevLayer* layers;
    const void* embed;    // [V][d] storage dtype, row-major
    const uint4* wlm;     // [V/16][d/KB][64]
    const float* g_final;
    const float* rope_cos;   // [ctx_pad][hd/2]
    const float* rope_sin;
    float* X;             // residual stream [16][d]
    void* A;              // norm-fed GEMM input (gain applied, not yet divided by the RMS), operand order, d columns
    float* ssq;           // [d/16][16] partial sums of squares of X rows
    void* Q_hi;           // [16][qdim]
    void* Q_lo;
    float* att_part;      // [units][G][16][hd+4]: numerator[hd], max, denominator, 2 pad; units <= n_slots*Hkv*max_chunks
    float* xch;           // [group of tiles][K range][tile of the group][16 rows][16 columns]: partial tiles of a stage
                          // whose workgroups share K ranges in pairs (sized for the stage with most tiles)
    int* xch_ticket;      // [kSplitTickets]: workgroups of the pair that have delivered their partials
    void* O;              // merged attention output, operand order, qdim columns
    void* H;              // SwiGLU output, operand order, F columns
    float* logits;        // [16][V]
    float* best_val;      // [lm_wgs][16]
    int* best_idx;
    PassResult* res;
};

}  // namespace amusd
