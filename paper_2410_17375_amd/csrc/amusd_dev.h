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

// Values that change from pass to pass live in device memory so that a
// captured launch sequence can be replayed unchanged.
struct PassParams {
    int L;             // cache length before the pass (ctx_len)
    int k;             // rows
    int force_accept;  // 1: prefill, every row is kept
    int keep_logits;   // 1: store fp32 logits
    int p_ctx;         // model's greedy token for position L
    int pad[3];
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
    void* kcache;        // [Hkv][ctx_pad][hd] elements
    void* vcache;        // [Hkv][ctx_pad/BK][hd/16][64 lanes][EPL] elements (matrix-core operand order)
};

struct DevModel {
    int n_layers, d, Hq, Hkv, hd, F, V, G;
    int qdim, kvdim, nqkv;
    int max_ctx, ctx_pad;
    int dtype;
    int chunk;            // keys per attention work unit (waves x keys-per-block)
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
    void* A_hi;           // GEMM input, gain applied, not yet divided by the RMS: [16][d] (bf16 hi part, or fp32)
    void* A_lo;           // bf16 lo part
    float* ssq;           // [d/16][16] partial sums of squares of X rows
    void* Q_hi;           // [16][qdim]
    void* Q_lo;
    float* att_part;      // [units][G][16][hd+4]: numerator[hd], max, denominator, 2 pad
    void* O_hi;           // merged attention output [16][qdim]
    void* O_lo;
    void* H_hi;           // SwiGLU output [16][F]
    void* H_lo;
    float* logits;        // [16][V]
    float* best_val;      // [lm_wgs][16]
    int* best_idx;
    const int* tokens;    // [16]
    const PassParams* pp;
    PassResult* res;
    unsigned* barrier;    // grid barrier state (single-kernel mode)
};

}  // namespace amusd
