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

// Per-pass values.  They travel as kernel arguments (no device round trip
// before the first weight load can be addressed).
struct PassArgs {
    int L;             // cache length before the pass (ctx_len)
    int k;             // rows
    int force_accept;  // 1: prefill, every row is kept
    int keep_logits;   // 1: store fp32 logits
    int p_ctx;         // model's greedy token for position L
    int tokens[kRows]; // input token of each row
};

struct PassResult {
    int accept_len;
    int next_token;
    int greedy[kRows];
    int pad[14];
};

struct DevLayer {
    const uint4* wqkv;   // fragment-ordered [ (Hq+2Hkv)*hd/16 tiles ][ d/KB ][64 lanes] x 16 B
    const uint4* wo;     // [d/16][qdim/KB][64]
    const uint4* wgu;    // [2F/16][d/KB][64]   tile t: rows 0-7 gate features 8t.., rows 8-15 up features 8t..
    const uint4* wd;     // [d/16][F/KB][64]
    const float* g_attn; // [d]
    const float* g_mlp;  // [d]
    void* kcache;        // [Hkv][ctx_pad/16][hd/4/EPL][64 lanes][EPL] elements (operand order of the score product)
    void* vcache;        // [Hkv][ctx_pad/BK][hd/16][64 lanes][EPL] elements (matrix-core operand order)
};

struct DevModel {
    int n_layers, d, Hq, Hkv, hd, F, V, G;
    int qdim, kvdim, nqkv;
    int max_ctx, ctx_pad;
    int dtype;
    int chunk;            // keys per attention work unit: (8/G) runs x bpw blocks x keys-per-block
    int bpw;              // key blocks a wave walks in one attention work unit
    int max_chunks;
    int lm_wgs;           // workgroups that produce arg-max partials
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
    float* att_part;      // [units][G][16][hd+4]: numerator[hd], max, denominator, 2 pad
    void* O;              // merged attention output, operand order, qdim columns
    void* H;              // SwiGLU output, operand order, F columns
    float* logits;        // [16][V]
    float* best_val;      // [lm_wgs][16]
    int* best_idx;
    PassResult* res;
    unsigned* barrier;    // grid barrier state (single-kernel mode)
};

}  // namespace amusd
