// HIP kernels of the verify pass for gfx950 (CDNA4, 64-wide waves).
//
// One pass = k <= 16 token rows through a Llama-style decoder against the
// key-value cache (VerifyTokens of Algorithm 1), greedy arg-max per row, and
// the longest-matching-prefix test.  The pass is bound by streaming the
// weights once from HBM, so the design is about keeping many 16-byte loads in
// flight and reading every weight byte exactly once:
//   * weights are stored in matrix-core operand order: a wave's load of one
//     16x32 (bf16) / 16x16 (fp32) weight fragment is 1 KiB contiguous;
//   * the k rows are padded to the 16-row MFMA tile, so a row's result does
//     not depend on k: a k-row pass equals k one-row passes bit for bit;
//   * a workgroup owns whole 16-column output tiles; its 8 waves split the
//     contraction dimension and reduce through LDS in a fixed order (no float
//     atomics anywhere), then run the fused epilogue (RMSNorm scale, rotary
//     embedding + cache append, SwiGLU, residual, arg-max partials);
//   * activations travel between stages as bf16 hi+lo pairs (x = hi + lo to
//     ~16 mantissa bits), so the bf16 MFMA path loses nothing on the
//     activation side; weights are exact bf16.
// Every stage is a __device__ function over (workgroup id, workgroup count),
// launched as one kernel per stage.
#include <hip/hip_ext.h>
#include <hip/hip_fp16.h>

#include "amusd_launch.h"

namespace amusd {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------- dtype traits
struct BF16 {
    static constexpr int EPL = 8;         // elements in a lane's 16-byte fragment
    static constexpr int KB = 32;         // contraction elements per fragment (4 lane groups x EPL)
    static constexpr int ESZ = 2;
    static constexpr int TPB = 2;         // 16-key score tiles per value block
    static constexpr int BLOCK_KEYS = 32;
    static constexpr bool HAS_LO = true;
    static __device__ __forceinline__ v4f mfma(uint4 a, uint4 b, v4f c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    }
    // Attention operands (cache, queries, probabilities) are IEEE half: the same 2 bytes per element as
    // bf16 with three more mantissa bits; their magnitudes (keys, values, queries O(1), probabilities
    // in [0,1]) sit well inside the half range, and stores clamp to it.
    static __device__ __forceinline__ v4f mfma_att(uint4 a, uint4 b, v4f c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t att_bits(float x) {
        const float c = fminf(fmaxf(x, -65504.f), 65504.f);
        return (uint32_t)__half_as_ushort(__float2half_rn(c));
    }
    static __device__ __forceinline__ float att_float(uint32_t b) { return __half2float(__ushort_as_half((unsigned short)b)); }
};
struct FP32 {
    static constexpr int EPL = 4;
    static constexpr int KB = 16;
    static constexpr int ESZ = 4;
    static constexpr int TPB = 1;
    static constexpr int BLOCK_KEYS = 16;
    static constexpr bool HAS_LO = false;
    static __device__ __forceinline__ v4f mfma(uint4 a, uint4 b, v4f c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ v4f mfma_att(uint4 a, uint4 b, v4f c) { return mfma(a, b, c); }
    static __device__ __forceinline__ uint32_t att_bits(float x) { return __float_as_uint(x); }
    static __device__ __forceinline__ float att_float(uint32_t b) { return __uint_as_float(b); }
};

__device__ __forceinline__ uint32_t bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// store a query element: fp32 as is; 16-bit models as hi + lo halves of the attention element type
template <class DT>
__device__ __forceinline__ void store_act(void* hi, void* lo, size_t idx, float x) {
    if constexpr (DT::HAS_LO) {
        uint32_t h = DT::att_bits(x);
        uint32_t l = DT::att_bits(x - DT::att_float(h));
        reinterpret_cast<uint16_t*>(hi)[idx] = (uint16_t)h;
        reinterpret_cast<uint16_t*>(lo)[idx] = (uint16_t)l;
    } else {
        reinterpret_cast<float*>(hi)[idx] = x;
    }
}

// GEMM inputs are kept in matrix-core operand order, so that a wave fetches the
// 16 rows x one K block it needs with ONE contiguous 1 KiB load, exactly like
// a weight fragment: buf[kb][part][lane = g*16 + slot][EPL elements], where g
// selects the lane group's EPL columns of the K block.
//   fp32        : one part, slot = row.
//   bf16, k <= 8: one part; slots 0-7 hold the hi halves of rows 0-7 and slots
//                 8-15 their lo halves (x = hi + lo), so one MFMA yields W.hi in
//                 result columns 0-7 and W.lo in columns 8-15;
//   bf16, k > 8 : two parts (hi, lo), slot = row.
// In both bf16 forms a wave adds its W.hi and W.lo sums before the cross-wave
// reduction, so a row's value does not depend on which form carried it.
template <class DT>
__device__ __forceinline__ void store_gemm_in(void* buf, int k_rows, int m, int col, float x) {
    const int kb = col / DT::KB, g = (col % DT::KB) / DT::EPL, e = col % DT::EPL;
    if constexpr (DT::HAS_LO) {
        const uint32_t h = bf16_rne(x);
        const uint32_t l = bf16_rne(x - bf16_to_f32(h));
        uint16_t* b = reinterpret_cast<uint16_t*>(buf);
        if (k_rows <= 8) {
            const size_t base = ((size_t)kb * 64 + g * 16 + m) * 8 + e;
            b[base] = (uint16_t)h;
            b[base + 8 * 8] = (uint16_t)l;                 // slot m + 8
        } else {
            const size_t base = ((size_t)kb * 128 + g * 16 + m) * 8 + e;
            b[base] = (uint16_t)h;
            b[base + 64 * 8] = (uint16_t)l;                // part 1
        }
    } else {
        reinterpret_cast<float*>(buf)[((size_t)kb * 64 + g * 16 + m) * 4 + e] = x;
    }
}

// Element index of key `pos`, head_dim column `c` in a kv head's key cache.  Keys are kept in the operand
// order of the score product: [16-key tile][fragment i][lane = g*16 + key%16][EPL], where lane group g owns
// columns g*hd/4 .. (g+1)*hd/4 and fragment i its i-th run of EPL columns, so a wave fetches one
// (tile, fragment) with a single contiguous 1 KiB load.
template <class DT>
__device__ __forceinline__ size_t kcache_index(int hd, int pos, int c) {
    const int q = hd / 4, g = c / q, w = c % q;
    return ((((size_t)(pos >> 4) * (q / DT::EPL) + w / DT::EPL) * 64) + g * 16 + (pos & 15)) * DT::EPL + w % DT::EPL;
}

// Weights are read once per pass: a non-temporal load keeps them from evicting
// the (re-read) activations from L2.
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

template <class DT>
__device__ __forceinline__ uint4 load_frag(const void* base, size_t elem_index) {
    return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + elem_index * DT::ESZ);
}

// Forces a (wave-uniform) kernel argument into a scalar register at this point of the program.  Left to itself
// the compiler loads an argument where it is first used, often behind a branch; a stage that starts by asking
// for everything it needs waits for argument memory once instead of several times in a row.
template <class T>
__device__ __forceinline__ void pin_scalar(const T& x) { asm volatile("" ::"s"(x)); }

// The value that lane (l ^ OFF) holds, without going through the LDS crossbar (`__shfl_xor` compiles to
// ds_bpermute, 50-100 clocks each, and these exchanges sit in chains on the critical path of every stage's end):
// data-parallel-primitive modifiers inside a row of 16 lanes, the gfx950 row and half-wave swaps across rows.
template <int OFF>
__device__ __forceinline__ uint32_t lane_xor_u(uint32_t v) {
    static_assert(OFF == 1 || OFF == 2 || OFF == 4 || OFF == 8 || OFF == 16 || OFF == 32, "one bit of the lane index");
    const int x = (int)v;
    if constexpr (OFF == 1) {
        return (uint32_t)__builtin_amdgcn_update_dpp(x, x, 0xB1, 0xf, 0xf, false);        // quad_perm:[1,0,3,2]
    } else if constexpr (OFF == 2) {
        return (uint32_t)__builtin_amdgcn_update_dpp(x, x, 0x4E, 0xf, 0xf, false);        // quad_perm:[2,3,0,1]
    } else if constexpr (OFF == 4) {
        const int t = __builtin_amdgcn_update_dpp(x, x, 0x104, 0xf, 0x5, false);          // row_shl:4 into lanes 0-3, 8-11
        return (uint32_t)__builtin_amdgcn_update_dpp(t, x, 0x114, 0xf, 0xa, false);       // row_shr:4 into lanes 4-7, 12-15
    } else if constexpr (OFF == 8) {
        return (uint32_t)__builtin_amdgcn_update_dpp(x, x, 0x128, 0xf, 0xf, false);       // row_ror:8
    } else if constexpr (OFF == 16) {
        const auto p = __builtin_amdgcn_permlane16_swap(v, v, false, false);   // p[0]: rows 0,0,2,2   p[1]: rows 1,1,3,3
        return (threadIdx.x & 16) ? p[0] : p[1];
    } else {
        const auto p = __builtin_amdgcn_permlane32_swap(v, v, false, false);   // p[0]: lanes 0-31 twice   p[1]: lanes 32-63 twice
        return (threadIdx.x & 32) ? p[0] : p[1];
    }
}
template <int OFF>
__device__ __forceinline__ float lane_xor(float v) { return __uint_as_float(lane_xor_u<OFF>(__float_as_uint(v))); }
template <int OFF>
__device__ __forceinline__ int lane_xor(int v) { return (int)lane_xor_u<OFF>((uint32_t)v); }
template <int OFF>
__device__ __forceinline__ float wave_xor_add(float v) { return v + lane_xor<OFF>(v); }
// all 64 lanes, offsets 32, 16, .., 1 in that order
__device__ __forceinline__ float wave_max_all(float v) {
    v = fmaxf(v, lane_xor<32>(v)); v = fmaxf(v, lane_xor<16>(v)); v = fmaxf(v, lane_xor<8>(v));
    v = fmaxf(v, lane_xor<4>(v)); v = fmaxf(v, lane_xor<2>(v)); v = fmaxf(v, lane_xor<1>(v));
    return v;
}
__device__ __forceinline__ float wave_sum_all(float v) {
    v = wave_xor_add<32>(v); v = wave_xor_add<16>(v); v = wave_xor_add<8>(v);
    v = wave_xor_add<4>(v); v = wave_xor_add<2>(v); v = wave_xor_add<1>(v);
    return v;
}
// lane j's value in every lane (j the same in all lanes)
__device__ __forceinline__ float lane_value(float v, int j) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), j));
}

// ---------------------------------------------------------------- RMS scale of the 16 rows
// The per-tile partial sums of squares are fetched at the start of a stage
// (so the fetch is the oldest entry of the load queue and never stalls the
// weight stream) and reduced in a fixed order just before the epilogue.
// The first use of the fetched values stays behind the contraction: an empty asm statement stops the compiler from
// moving the loop-invariant sum in front of the round loop, where the wave would wait for the values before it
// has asked for its first weights (0.4-0.5 us per launch on each of the three stages that use it).
// Only the first wave of each SIMD (waves 0-3) does this work, for the rows the pass has: those waves finish their
// K share well before their SIMD's second wave, so the chain of dependent shuffles, the division and the root
// (0.45 us) run while the others still stream, instead of after the last of them.
// Thread (row m = tid/32 and m + 8, slot s = tid%32) of waves 0-3 sums tiles s, s+32, ..
struct RstdPrefetch {
    static constexpr int N = 8;      // covers d <= 4096 from registers; larger d loops in finish()
    float v[2][N];
    int k_rows;
    __device__ __forceinline__ void begin(const DevModel& M, int rows) {
        k_rows = rows;
        if (threadIdx.x >= kThreads / 2) return;
        const int s = threadIdx.x & 31;
        const int ntp = M.d / 16;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int m = (threadIdx.x >> 5) + 8 * h;
            if (m < k_rows) {
#pragma unroll
                for (int t = 0; t < N; ++t) {
                    const int idx = s + 32 * t;
                    v[h][t] = M.ssq[(idx < ntp ? idx : ntp - 1) * kRows + m];
                }
            }
        }
    }
    __device__ __forceinline__ void finish(const DevModel& M, float* rstd) {
        if (threadIdx.x >= kThreads / 2) return;
        const int s = threadIdx.x & 31;
        const int ntp = M.d / 16;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int m = (threadIdx.x >> 5) + 8 * h;
            if (m < k_rows) {
                float acc = 0.f;
#pragma unroll
                for (int t = 0; t < N; ++t) {
                    float x = v[h][t];
                    asm volatile("" : "+v"(x));
                    acc += s + 32 * t < ntp ? x : 0.f;
                }
                for (int idx = s + 32 * N; idx < ntp; idx += 32) acc += M.ssq[idx * kRows + m];
                acc = wave_xor_add<16>(acc);
                acc = wave_xor_add<8>(acc);
                acc = wave_xor_add<4>(acc);
                acc = wave_xor_add<2>(acc);
                acc = wave_xor_add<1>(acc);
                if (s == 0) rstd[m] = 1.0f / sqrtf(acc / (float)M.d + M.eps);
            }
        }
    }
};

// ---------------------------------------------------------------- LDS layout (dynamic shared memory, floats)
constexpr int kAttPad = 4;    // row padding of the attention partials (spreads LDS banks)
constexpr int kScratchFloats = kWaves * kRows * (128 + kAttPad) + kWaves * kRows * 2;   // attention partials; >= GEMM reduction area
static_assert(kScratchFloats >= kWaves * kMaxTilesPerRound * 256, "GEMM reduction area must fit");
constexpr int kOffRstd = kScratchFloats;
constexpr int kOffTileBestV = kOffRstd + kRows;
constexpr int kOffTileBestI = kOffTileBestV + kMaxTilesPerRound * kRows;
constexpr int kOffPfSink = kOffTileBestI + kMaxTilesPerRound * kRows;   // per wave, 64 words nobody reads
constexpr int kSmemFloats = kOffPfSink + kWaves * 64;

// ---------------------------------------------------------------- skinny GEMM stage
// C[n][m] = sum_k W[n][k] * A[m][k] for the 16 rows m, output tiles of 16
// columns n.  Workgroup wg owns tiles wg, wg+nwg, ...; up to 8 per round.
// Wave w contracts over its slice of the K blocks; partial tiles are summed
// through LDS in wave order, then epi.item() runs on every pair
// (column r, column r+8) of each tile.
//
// The contraction loop is a software pipeline of D stages, one stage = one K
// block = NT weight fragments + the activation fragment(s).  All loads are
// unconditional (out-of-range stages re-read the last stage and multiply by a
// zeroed activation), so the loop body is straight-line code and the hardware
// load queue stays D stages deep: with 8 waves per CU that is 64-128 KiB of
// weight bytes in flight per CU, what it takes to cover HBM latency.  Deeper is
// not better: one- and two-tile rounds carry as many activation bytes as weight
// bytes through the same queue, and measured fastest 8 KiB of weights deep per
// wave (D = 8 and 4; 16 and 8 cost the down projection 1.1 us per launch, and a
// bare streaming kernel is faster at 8 loads in flight per wave than at 16 or 24).
//
// A wave walks its K blocks from a start that depends on (workgroup, wave) and
// wraps around (`rot`): 2048 waves that all begin at the first block of their
// slice march through addresses that differ only in high bits and crowd the
// same memory channels; staggered starts measured 3-4 % faster on the large
// stages.  The order of a wave's additions depends on the workgroup and wave
// only, never on k or on the position, so results stay independent of those.
enum { kActSingle = 0, kActPacked8 = 1, kActHiLo = 2 };
constexpr int kAttPf = 12;        // O-projection weight fragments (1 KiB) per wave fetched ahead by the attention stage
constexpr int kAttPfMax = 3;      // O-projection workgroups served by one idle attention workgroup, at most
constexpr int kAttPfSleep = 0;    // s_sleep units (64 clocks) before the fetch (0: at once; the units find their cache rows in L2)
constexpr size_t kKvPrefetchMax = 2u << 20;   // cache bytes per XCD up to which they do (context 4096 at the 8B shape)
constexpr bool kKvPrefetch = true; // QKV workgroups with time to spare fetch the cache rows the attention stage reads next

template <class DT, int MODE, int NT, int D>
__device__ __forceinline__ void gemm_accumulate(v4f (&out)[kMaxTilesPerRound], const uint4* __restrict__ W, int tile0,
                                                int tile_stride, int kblocks, int kb0, int S, int rot, int kstride,
                                                const uint4* __restrict__ act, int lane) {
    auto blk = [&](int st) { const int x = st + rot; return (x >= S ? x - S : x) * kstride; };   // stage -> K block, from kb0
    constexpr int AF = MODE == kActHiLo ? 2 : 1;          // activation fragments per K block
    v4f acc[NT * AF];
#pragma unroll
    for (int j = 0; j < NT * AF; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
    const uint4* wp[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) wp[j] = W + ((size_t)(tile0 + tile_stride * j) * kblocks + kb0) * 64 + lane;
    const uint4* ap = act + (size_t)kb0 * (AF * 64) + lane;
    uint4 wb[D][NT], ab[D][AF];
    const int last = S - 1;
#pragma unroll
    for (int i = 0; i < D; ++i) {
        const int s = blk(i < last ? i : last);
#pragma unroll
        for (int j = 0; j < NT; ++j) wb[i][j] = load_stream(wp[j] + (size_t)s * 64);
#pragma unroll
        for (int f = 0; f < AF; ++f) ab[i][f] = ap[(size_t)s * (AF * 64) + f * 64];
        __builtin_amdgcn_sched_barrier(0);   // same issue order as in the loop: the loop's waits are sized for it
    }
    int s0 = 0;
    for (; s0 + D < S; s0 += D) {
#pragma unroll
        for (int i = 0; i < D; ++i) {
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int f = 0; f < AF; ++f) acc[j * AF + f] = DT::mfma(wb[i][j], ab[i][f], acc[j * AF + f]);
            const int sn = blk(s0 + i + D < last ? s0 + i + D : last);
#pragma unroll
            for (int j = 0; j < NT; ++j) wb[i][j] = load_stream(wp[j] + (size_t)sn * 64);
#pragma unroll
            for (int f = 0; f < AF; ++f) ab[i][f] = ap[(size_t)sn * (AF * 64) + f * 64];
            // Keep the stages in this order.  Left alone, the scheduler gathers the matrix instructions of all D
            // stages first and all loads behind them, so a wave waits for its whole queue at the top of the loop
            // and has nothing in flight while it computes.
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int i = 0; i < D; ++i) {
        const bool on = s0 + i < S;
        const uint4 z = uint4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int f = 0; f < AF; ++f) acc[j * AF + f] = DT::mfma(wb[i][j], on ? ab[i][f] : z, acc[j * AF + f]);
    }
    // The wave's W.hi and W.lo sums are added here, in one fixed order for every k: two accumulators of a
    // tile (kActHiLo), or result columns m and m+8 of one accumulator (kActPacked8; lanes m < 8 keep the sum).
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        if constexpr (MODE == kActHiLo) {
            out[j] = acc[2 * j] + acc[2 * j + 1];
        } else if constexpr (MODE == kActPacked8) {
            v4f lo;
            lo.x = lane_xor<8>(acc[j].x);
            lo.y = lane_xor<8>(acc[j].y);
            lo.z = lane_xor<8>(acc[j].z);
            lo.w = lane_xor<8>(acc[j].w);
            out[j] = acc[j] + lo;
        } else {
            out[j] = acc[j];
        }
    }
}

// A wave's share of the K blocks of a GEMM stage, and where in it the wave starts its walk: blocks
// kb0 + stride * ((i + rot) mod S), i = 0 .. S-1.
// K split: SIMD s hosts waves s and s+4; they share the K quarter of their SIMD, the first of them taking
// old_share sixteenths (the first wave of a SIMD wins the issue arbitration and streams faster, but which split is
// fastest was measured per stage, and it also shifts where the second wave's stream starts).
// Interleaved form: the waves take every eighth block instead (the two waves of a SIMD neighbouring ones), so that a
// workgroup's eight streams move through the tile as one window of 8 KiB.
struct KSlice {
    int kb0, S, rot, stride;
};
__device__ __forceinline__ KSlice k_slice(int kblocks, int wg, int wave, bool stagger, int rot_wg, int rot_wave,
                                          bool interleave, int old_share) {
    const int simd = wave & 3, young = wave >> 2;
    const int q0 = (kblocks * simd) / 4, q1 = (kblocks * (simd + 1)) / 4;
    const int cut = q0 + ((q1 - q0) * old_share + 8) / 16;
    KSlice k;
    k.kb0 = young ? cut : q0;
    k.S = (young ? q1 : cut) - k.kb0;
    k.stride = 1;
    if (interleave) {
        k.kb0 = simd * 2 + young;
        k.S = (kblocks - k.kb0 + kWaves - 1) / kWaves;
        k.stride = kWaves;
    }
    k.rot = stagger && k.S > 0 ? (int)(((unsigned)wg * (unsigned)rot_wg + (unsigned)wave * (unsigned)rot_wave) % (unsigned)k.S) : 0;
    return k;
}
__device__ __forceinline__ int round_tiles(int left) { return left >= 8 ? 8 : left == 7 ? 7 : left >= 4 ? 4 : left >= 2 ? 2 : 1; }

// Weights of a GEMM stage that runs later in the pass, fetched into L2 ahead of time.  The L2 of an XCD keeps what
// its workgroups have read across kernel boundaries, and workgroup w of every stage runs on the same XCD
// (w mod 8): reading one word of each 128-byte line of the fragments that workgroup wg of the later stage will
// stream puts them where that workgroup will find them.  This only pays where the memory system would
// otherwise sit idle (the attention stage waits on latency, not on bytes); between two streaming
// stages it just moves bytes from one kernel to the other, and measured slower.  Weights are never written after
// the model is loaded, so a line fetched early can never be stale.
struct NextWeights {
    const uint4* W;
    int n_tiles, kblocks;
    bool stagger;
    int rot_wg, rot_wave;   // the consumer's K-walk coefficients (k_slice)
    bool interleave;
    int old_share;
};
// Fragments [F0, F1) of consumer wave `cwave`, counted in the order the consumer's pipeline asks for them
// (stage-major over the tiles of its first round); 8 fragments (8 KiB) per load instruction of the calling wave.
// The loads deliver straight into LDS (64 words per wave that nobody reads), so they need no result registers.
template <int F0, int F1>
__device__ __forceinline__ void prefetch_frags(const NextWeights& nx, int wg, int nwg, int cwave, int lane, float* lds_sink) {
    if (F1 <= F0 || wg >= nx.n_tiles) return;
    const KSlice ks = k_slice(nx.kblocks, wg, cwave, nx.stagger, nx.rot_wg, nx.rot_wave, nx.interleave, nx.old_share);
    if (ks.S <= 0) return;
    const int nt = round_tiles((nx.n_tiles - wg + nwg - 1) / nwg);
#pragma unroll
    for (int f0 = F0; f0 < F1; f0 += 8) {
        const int f = f0 + (lane >> 3), q = lane & 7;
        const int ff = f < F1 ? f : F1 - 1;                // lanes beyond the last fragment repeat it
        const int i = ff / nt, j = ff % nt;
        const int x = (i < ks.S ? i : ks.S - 1) + ks.rot;
        const int blk = (x >= ks.S ? x - ks.S : x) * ks.stride;
        const char* p = reinterpret_cast<const char*>(nx.W + ((size_t)(wg + nwg * j) * nx.kblocks + ks.kb0 + blk) * 64) + q * 128;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                         (__attribute__((address_space(3))) void*)lds_sink, 4, 0, 0);
    }
}
// A wave must not end while a load is in flight.
__device__ __forceinline__ void prefetch_retire() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// MODE as above.  A wave hands one partial tile per output tile to the reduction, whatever the mode.
template <class DT, int MODE, class Epi>
__device__ __forceinline__ void gemm_stage_m(const uint4* __restrict__ W, int n_tiles, int kblocks,
                                             const void* __restrict__ A, int wg, int nwg, Epi& epi, float* smem) {
    constexpr int SLOTS = kMaxTilesPerRound;                  // partial tiles per wave per round
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const KSlice ks = k_slice(kblocks, wg, wave, Epi::kStagger, Epi::kRotWg, Epi::kRotWave, Epi::kInterleave, Epi::kOldShare);
    const int kb0 = ks.kb0, S = ks.S, rot = ks.rot;
    const int mine = wg < n_tiles ? (n_tiles - wg + nwg - 1) / nwg : 0;
    const uint4* act = reinterpret_cast<const uint4*>(A);
    bool first = true;
    for (int i0 = 0; i0 < mine;) {
        const int left = mine - i0;
        const int nt = round_tiles(left);
        const int t0 = wg + nwg * i0;
        epi.prefetch(t0, nwg, nt);
        v4f acc[SLOTS];
#pragma unroll
        for (int j = 0; j < SLOTS; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
        if (S > 0) {
            if constexpr (MODE == kActHiLo) {
                switch (nt) {
                    case 8: gemm_accumulate<DT, MODE, 8, 2>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    case 7: gemm_accumulate<DT, MODE, 7, 2>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    case 4: gemm_accumulate<DT, MODE, 4, 3>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    case 2: gemm_accumulate<DT, MODE, 2, 4>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    default: gemm_accumulate<DT, MODE, 1, 4>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                }
            } else {
                switch (nt) {
                    case 8: gemm_accumulate<DT, MODE, 8, 2>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    case 7: gemm_accumulate<DT, MODE, 7, 2>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    case 4: gemm_accumulate<DT, MODE, 4, 4>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    case 2: gemm_accumulate<DT, MODE, 2, 4>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                    default: gemm_accumulate<DT, MODE, 1, 8>(acc, W, t0, nwg, kblocks, kb0, S, rot, ks.stride, act, lane); break;
                }
            }
        }
        // partial tiles to LDS as [wave][slot][column m][n]; lane holds n = 4g..4g+3 of result column m
        // (kActPacked8: columns 8..15 carry nothing the reduction reads)
#pragma unroll
        for (int j = 0; j < SLOTS; ++j)
            if (j < nt && (MODE != kActPacked8 || m < 8))
                *reinterpret_cast<v4f*>(smem + ((wave * SLOTS + j) * 256 + m * 16 + g * 4)) = acc[j];
        if (first) epi.prepare();
        __syncthreads();
#pragma unroll
        for (int it = 0; it * kThreads < SLOTS * 128; ++it) {
            const int item = tid + it * kThreads;
            const int j = item >> 7, mm = (item >> 3) & 15, r = item & 7;
            const bool valid = j < nt && (MODE != kActPacked8 || mm < 8);
            float v1 = 0.f, v2 = 0.f;
            if (valid) {
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    v1 += smem[(w * SLOTS + j) * 256 + mm * 16 + r];
                    v2 += smem[(w * SLOTS + j) * 256 + mm * 16 + r + 8];
                }
            }
            epi.item(t0 + nwg * (valid ? j : 0), j, it, mm, r, v1, v2, valid);
        }
        __syncthreads();
        epi.round_end(nt);
        first = false;
        i0 += nt;
    }
}

template <class DT, class Epi>
__device__ __forceinline__ void gemm_stage(const uint4* __restrict__ W, int n_tiles, int kblocks,
                                           const void* __restrict__ A, int k_rows, int wg, int nwg, Epi& epi,
                                           float* smem) {
    if constexpr (!DT::HAS_LO) {
        gemm_stage_m<DT, kActSingle>(W, n_tiles, kblocks, A, wg, nwg, epi, smem);
    } else {
        if (k_rows <= 8) gemm_stage_m<DT, kActPacked8>(W, n_tiles, kblocks, A, wg, nwg, epi, smem);
        else gemm_stage_m<DT, kActHiLo>(W, n_tiles, kblocks, A, wg, nwg, epi, smem);
    }
}

// ---------------------------------------------------------------- K split over a pair of workgroups
// Words that one workgroup writes and a workgroup on another compute unit reads inside the same kernel: every
// access is a relaxed atomic at device scope, which the hardware carries out past the caches that are private to
// a compute unit or to one of the chip's eight dies.
__device__ __forceinline__ void store_shared_f(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_shared_f(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// WAYS workgroups share the work on NT tiles, each contracting over one WAYS-th of the K blocks: with G groups of NT
// tiles, workgroup p * G + g takes the p-th K range of tiles g, g + G, ...  Each writes its partial tiles to device
// memory and counts itself; whichever counts last adds the partials in the order of the K ranges (its own from
// registers, so the bits do not depend on who is last) and runs the epilogue.  Nobody waits for anybody.  kblocks is
// a multiple of WAYS and n_tiles of NT (the host checks).
//   NT = 1, WAYS = 2: a stage with tiles for at most half the compute units and a long contraction (the down
//           projection of a narrow model) leaves half the chip without work, and what one compute unit can pull
//           through its load path then bounds the stage; the split puts every compute unit to work.
//   NT = WAYS = 2: a stage with one tile per compute unit moves as many activation bytes as weight bytes through each
//           compute unit's load path; two tiles over half the K range need half the activation bytes per weight byte.
//           (Four tiles over a quarter of the K range measured no faster than no split at all: the last of four
//           workgroups to finish has three partials to wait for and add.)
template <class DT, int MODE, int NT, int WAYS, class Epi>
__device__ __forceinline__ bool gemm_stage_split_m(const uint4* __restrict__ W, int n_tiles, int kblocks,
                                                   const void* __restrict__ A, int wg, Epi& epi, float* smem,
                                                   float* xch, int* ticket) {
    static_assert(WAYS <= kSplitWaysMax, "the exchange buffer holds kSplitWaysMax partial tiles per tile");
    constexpr int SLOTS = kMaxTilesPerRound;
    constexpr int D = NT == 1 ? (MODE == kActHiLo ? 4 : 8) : NT >= 4 && MODE == kActHiLo ? 3 : 4;   // as in gemm_stage_m
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int groups = n_tiles / NT;
    const int grp = wg % groups, part = wg / groups;
    const int kh = kblocks / WAYS;
    const KSlice ks = k_slice(kh, wg, wave, Epi::kStagger, Epi::kRotWg, Epi::kRotWave, Epi::kInterleave, Epi::kOldShare);
    const uint4* act = reinterpret_cast<const uint4*>(A);
    epi.prefetch(grp, groups, NT);
    v4f acc[SLOTS];
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
    if (ks.S > 0) gemm_accumulate<DT, MODE, NT, D>(acc, W, grp, groups, kblocks, ks.kb0 + part * kh, ks.S, ks.rot, ks.stride, act, lane);
#pragma unroll
    for (int j = 0; j < NT; ++j)
        if (MODE != kActPacked8 || m < 8) *reinterpret_cast<v4f*>(smem + ((wave * SLOTS + j) * 256 + m * 16 + g * 4)) = acc[j];
    epi.prepare();
    __syncthreads();
    const int j = tid >> 7, mm = (tid >> 3) & 15, r = tid & 7;             // thread -> (tile of the group, row, column pair)
    const bool valid = j < NT && (MODE != kActPacked8 || mm < 8);
    float v1 = 0.f, v2 = 0.f;
    if (valid) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            v1 += smem[(w * SLOTS + j) * 256 + mm * 16 + r];
            v2 += smem[(w * SLOTS + j) * 256 + mm * 16 + r + 8];
        }
        float* mine = xch + (((size_t)grp * WAYS + part) * NT + j) * 256;
        store_shared_f(mine + mm * 16 + r, v1);
        store_shared_f(mine + mm * 16 + r + 8, v2);
    }
    // the partials are complete in device memory once every wave's stores have been acknowledged; then they are counted
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int* s_flag = reinterpret_cast<int*>(smem + kOffTileBestI);
    if (tid == 0) {
        const int seen = __hip_atomic_fetch_add(ticket + grp, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen == WAYS - 1) __hip_atomic_store(ticket + grp, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next layer
        *s_flag = seen == WAYS - 1;
    }
    __syncthreads();
    if (!*s_flag) return false;               // another workgroup of the group finishes the tiles
    if (valid) {
        float o1[WAYS], o2[WAYS];
#pragma unroll
        for (int p = 0; p < WAYS; ++p) {      // all loads first: one round trip
            const float* other = xch + (((size_t)grp * WAYS + p) * NT + j) * 256;
            o1[p] = load_shared_f(other + mm * 16 + r);
            o2[p] = load_shared_f(other + mm * 16 + r + 8);
        }
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int p = 0; p < WAYS; ++p) {      // K ranges in order; this workgroup's own partial from its registers
            s1 += p == part ? v1 : o1[p];
            s2 += p == part ? v2 : o2[p];
        }
        v1 = s1;
        v2 = s2;
    }
    epi.item(grp + groups * (valid ? j : 0), j, 0, mm, r, v1, v2, valid);
    __syncthreads();
    epi.round_end(NT);
    return true;
}

// Returns true in the workgroup that finished the tiles (ran the epilogue), false in the one that was first.
template <class DT, int NT, int WAYS, class Epi>
__device__ __forceinline__ bool gemm_stage_split(const uint4* __restrict__ W, int n_tiles, int kblocks,
                                                 const void* __restrict__ A, int k_rows, int wg, Epi& epi, float* smem,
                                                 float* xch, int* ticket) {
    if constexpr (!DT::HAS_LO) {
        return gemm_stage_split_m<DT, kActSingle, NT, WAYS>(W, n_tiles, kblocks, A, wg, epi, smem, xch, ticket);
    } else {
        if (k_rows <= 8) return gemm_stage_split_m<DT, kActPacked8, NT, WAYS>(W, n_tiles, kblocks, A, wg, epi, smem, xch, ticket);
        return gemm_stage_split_m<DT, kActHiLo, NT, WAYS>(W, n_tiles, kblocks, A, wg, epi, smem, xch, ticket);
    }
}

// ---------------------------------------------------------------- epilogues
// An epilogue sees every pair (column r, column r+8) of each finished tile:
//   prefetch(t0, stride, nt)  before the contraction of a round (tiles t0 + stride*j, j < nt):
//                             fetch what item() will need, so it is the oldest entry of the load queue;
//   prepare()                 once, before the first round's items (may use LDS; a barrier follows);
//   item(tile, slot, it, row, r, v1, v2, valid)  thread's it-th item of the round (it < 2);
//   round_end(nt)             after the barrier that ends a round.

// thread's it-th item of a round -> (tile slot j, row, column pair r)
__device__ __forceinline__ void item_coords(int it, int& j, int& mm, int& r) {
    const int item = threadIdx.x + it * kThreads;
    j = item >> 7;
    mm = (item >> 3) & 15;
    r = item & 7;
}

// Residual update for a pair of columns, then the next GEMM's input x*gain
// (in operand order) and the tile's partial sum of squares per row.
template <class DT>
__device__ __forceinline__ void residual_pair(const DevModel& M, float g1, float g2, int tile, int mm, int r, float x1,
                                              float x2, int k_rows, bool on) {
    const int c1 = tile * 16 + r, c2 = c1 + 8;
    float sq = 0.f;
    if (on) {
        M.X[(size_t)mm * M.d + c1] = x1;
        M.X[(size_t)mm * M.d + c2] = x2;
        store_gemm_in<DT>(M.A, k_rows, mm, c1, x1 * g1);
        store_gemm_in<DT>(M.A, k_rows, mm, c2, x2 * g2);
        sq = x1 * x1 + x2 * x2;
    }
    sq = wave_xor_add<1>(sq);
    sq = wave_xor_add<2>(sq);
    sq = wave_xor_add<4>(sq);
    if (on && r == 0) M.ssq[tile * kRows + mm] = sq;
}

template <class DT, int STAGE>
struct EpiResidual {   // O-projection and down-projection: X += C, feed the next norm
    static constexpr int kStage = STAGE;
    static constexpr bool kStagger = true;
    // Where a wave starts its K walk (k_slice), swept per stage on the chip: the down projection is fastest when
    // all workgroups start alike and only the waves differ, the O-projection when nobody is shifted by its wave.
    static constexpr int kRotWg = STAGE == 6 ? 0 : 5, kRotWave = STAGE == 6 ? 5 : 0;
    static constexpr bool kInterleave = STAGE == 6;   // down projection: 0.4 us per launch faster; the other stages equal or slower
    static constexpr int kOldShare = 8;
    const DevModel& M;
    const float* gain_next;
    int k_rows;
    float px1[2], px2[2], pg1[2], pg2[2];
    __device__ __forceinline__ void prefetch(int t0, int stride, int nt) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            int j, mm, r;
            item_coords(it, j, mm, r);
            px1[it] = px2[it] = pg1[it] = pg2[it] = 0.f;
            if (j < nt && mm < k_rows) {
                const int c1 = (t0 + stride * j) * 16 + r;
                px1[it] = M.X[(size_t)mm * M.d + c1];
                px2[it] = M.X[(size_t)mm * M.d + c1 + 8];
                pg1[it] = gain_next[c1];
                pg2[it] = gain_next[c1 + 8];
            }
        }
    }
    __device__ __forceinline__ void item(int tile, int /*slot*/, int it, int mm, int r, float v1, float v2, bool valid) {
        const bool on = valid && mm < k_rows;
        residual_pair<DT>(M, pg1[it], pg2[it], tile, mm, r, px1[it] + v1, px2[it] + v2, k_rows, on);
    }
    __device__ __forceinline__ void prepare() {}
    __device__ __forceinline__ void round_end(int) {}
};

// ONE: the pass holds one sequence, so a row's position and cache follow from three scalars next to k; otherwise
// they are looked up per row in the argument tables (dependent loads of argument memory).
template <class DT, bool ONE>
struct EpiQKV {
    static constexpr int kStage = 1;        // RMS scale, rotary embedding on (i, i+hd/2) pairs, Q to its buffer, K/V appended to the cache
    static constexpr bool kStagger = false; // measured slower with staggered K walks (short slices, two tile counts)
    static constexpr int kRotWg = 0, kRotWave = 0;
    static constexpr bool kInterleave = false;
    static constexpr int kOldShare = 6;     // 12 + 20 of a SIMD's 32 K blocks: 0.4 us per launch faster than 16 + 16 (10 likewise; 4, 12, odd values not)
    const DevModel& M;
    const DevLayer& Ly;
    float* rstd;         // LDS
    const PassArgs& P;
    int k_rows;
    RstdPrefetch pre;
    float pc[2], ps[2];
    // Position and cache of this thread's row (both items of a thread belong to the same row).  The 16-bit form
    // keeps them in two registers from the start of the kernel (0.5 us per launch faster than looking them up where
    // they are used); the fp32 form's contraction loop has no register left for that and looks them up.
    static constexpr bool kKeepRow = DT::HAS_LO;
    int pos_, slot_;
    __device__ __forceinline__ int lookup_pos(int mm) const {
        if constexpr (ONE) return P.L0 + mm;
        else return P.row_pos[mm];
    }
    __device__ __forceinline__ int lookup_slot(int mm) const {
        if constexpr (ONE) return P.slot0;
        else return P.seg[P.row_seg[mm]].slot;
    }
    __device__ __forceinline__ void begin() {
        if constexpr (kKeepRow) {
            const int mm = (threadIdx.x >> 3) & 15;
            pos_ = lookup_pos(mm);
            slot_ = lookup_slot(mm);
        }
        pre.begin(M, k_rows);
    }
    __device__ __forceinline__ int row_pos(int mm) const { return kKeepRow ? pos_ : lookup_pos(mm); }
    __device__ __forceinline__ int row_slot(int mm) const { return kKeepRow ? slot_ : lookup_slot(mm); }
    __device__ __forceinline__ void prefetch(int t0, int stride, int nt) {
        const int hd = M.hd, tph = hd / 16, rot_tiles = (M.qdim + M.kvdim) / 16;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            int j, mm, r;
            item_coords(it, j, mm, r);
            pc[it] = 1.f;
            ps[it] = 0.f;
            const int tile = t0 + stride * j;
            if (j < nt && mm < k_rows && tile < rot_tiles) {
                const int i = (tile % tph) * 8 + r;           // q and k sections both start at a head boundary
                const int pos = row_pos(mm);
                pc[it] = M.rope_cos[(size_t)pos * (hd / 2) + i];
                ps[it] = M.rope_sin[(size_t)pos * (hd / 2) + i];
            }
        }
    }
    __device__ __forceinline__ void prepare() { pre.finish(M, rstd); }
    __device__ __forceinline__ void item(int tile, int /*slot*/, int it, int mm, int r, float v1, float v2, bool valid) {
        if (!valid || mm >= k_rows) return;
        const int hd = M.hd, tph = hd / 16;
        const float sc = rstd[mm];
        const float x1 = v1 * sc, x2 = v2 * sc;
        const int pos = row_pos(mm);
        const size_t slot_base = (size_t)row_slot(mm) * M.Hkv * M.ctx_pad * hd;   // elements, K and V alike
        const int qt = M.qdim / 16, kt = M.kvdim / 16;
        if (tile < qt + kt) {
            const bool isq = tile < qt;
            const int tt = isq ? tile : tile - qt;
            const int head = tt / tph, i = (tt % tph) * 8 + r;
            const float c = pc[it], sn = ps[it];
            const float y1 = x1 * c - x2 * sn, y2 = x1 * sn + x2 * c;
            if (isq) {
                const size_t o = (size_t)mm * M.qdim + head * hd + i;
                store_act<DT>(M.Q_hi, M.Q_lo, o, y1);
                store_act<DT>(M.Q_hi, M.Q_lo, o + hd / 2, y2);
            } else {
                const size_t hb = slot_base + (size_t)head * M.ctx_pad * hd;
                const size_t o1 = hb + kcache_index<DT>(hd, pos, i), o2 = hb + kcache_index<DT>(hd, pos, i + hd / 2);
                if constexpr (DT::HAS_LO) {
                    reinterpret_cast<uint16_t*>(Ly.kcache)[o1] = (uint16_t)DT::att_bits(y1);
                    reinterpret_cast<uint16_t*>(Ly.kcache)[o2] = (uint16_t)DT::att_bits(y2);
                } else {
                    reinterpret_cast<float*>(Ly.kcache)[o1] = y1;
                    reinterpret_cast<float*>(Ly.kcache)[o2] = y2;
                }
            }
        } else {
            const int tt = tile - qt - kt;
            const int head = tt / tph, j = tt % tph;   // value features j*16 + r and j*16 + r + 8
            constexpr int BK = DT::BLOCK_KEYS;
            const int b = pos / BK, q = pos % BK;
            const int e = (q / 16) * 4 + (q % 4), gg = (q % 16) / 4;
            const size_t blk = ((size_t)head * (M.ctx_pad / BK) + b) * tph + j;
            const size_t o1 = slot_base + (blk * 64 + gg * 16 + r) * DT::EPL + e;
            const size_t o2 = slot_base + (blk * 64 + gg * 16 + r + 8) * DT::EPL + e;
            if constexpr (DT::HAS_LO) {
                reinterpret_cast<uint16_t*>(Ly.vcache)[o1] = (uint16_t)DT::att_bits(x1);
                reinterpret_cast<uint16_t*>(Ly.vcache)[o2] = (uint16_t)DT::att_bits(x2);
            } else {
                reinterpret_cast<float*>(Ly.vcache)[o1] = x1;
                reinterpret_cast<float*>(Ly.vcache)[o2] = x2;
            }
        }
    }
    __device__ __forceinline__ void round_end(int) {}
};

template <class DT>
struct EpiSwiGLU {     // tile rows 0-7 are gate features, 8-15 the matching up features
    static constexpr int kStage = 5;
    static constexpr bool kStagger = true;
    static constexpr int kRotWg = 5, kRotWave = 11;   // an even wave coefficient costs 0.3-6 us per launch
    static constexpr bool kInterleave = false;
    static constexpr int kOldShare = 8;
    const DevModel& M;
    float* rstd;
    int k_rows;
    RstdPrefetch pre;
    __device__ __forceinline__ void prefetch(int, int, int) {}
    __device__ __forceinline__ void prepare() { pre.finish(M, rstd); }
    __device__ __forceinline__ void item(int tile, int /*slot*/, int /*it*/, int mm, int r, float v1, float v2, bool valid) {
        if (!valid || mm >= k_rows) return;
        const float sc = rstd[mm];
        const float gate = v1 * sc, up = v2 * sc;
        const float h = gate / (1.0f + __expf(-gate)) * up;
        store_gemm_in<DT>(M.H, k_rows, mm, tile * 8 + r, h);
    }
    __device__ __forceinline__ void round_end(int) {}
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }
// keeps the better of this lane's (value, index) and lane (l ^ OFF)'s
template <int OFF>
__device__ __forceinline__ void keep_better_xor(float& bv, int& bi) {
    const float ov = lane_xor<OFF>(bv);
    const int oi = lane_xor<OFF>(bi);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
}

struct EpiLMHead {
    static constexpr int kStage = 7;     // logits (optionally stored); per-row arg-max over this workgroup's tiles, lowest id on ties
    static constexpr bool kStagger = true;
    static constexpr int kRotWg = 5, kRotWave = 11;
    static constexpr bool kInterleave = false;
    static constexpr int kOldShare = 8;
    const DevModel& M;
    float* smem;
    int k_rows, keep;
    float run_v;         // thread mm < 16 keeps the workgroup's running best for row mm
    int run_i;
    RstdPrefetch pre;
    __device__ __forceinline__ void prefetch(int, int, int) {}
    __device__ __forceinline__ void prepare() { pre.finish(M, smem + kOffRstd); }
    __device__ __forceinline__ void item(int tile, int slot, int /*it*/, int mm, int r, float v1, float v2, bool valid) {
        const float sc = smem[kOffRstd + mm];
        const float z1 = v1 * sc, z2 = v2 * sc;
        const int c1 = tile * 16 + r, c2 = c1 + 8;
        const bool on = valid && mm < k_rows;
        if (on && keep) {
            M.logits[(size_t)mm * M.V + c1] = z1;
            M.logits[(size_t)mm * M.V + c2] = z2;
        }
        float bv = on ? z1 : -INFINITY;
        int bi = on ? c1 : 0x7fffffff;
        if (on && better(z2, c2, bv, bi)) { bv = z2; bi = c2; }
        keep_better_xor<1>(bv, bi);                  // the 8 lanes of one (tile,row) are adjacent
        keep_better_xor<2>(bv, bi);
        keep_better_xor<4>(bv, bi);
        if (r == 0) {
            smem[kOffTileBestV + slot * kRows + mm] = bv;
            reinterpret_cast<int*>(smem)[kOffTileBestI + slot * kRows + mm] = bi;
        }
    }
    __device__ __forceinline__ void round_end(int nt) {   // called after a barrier
        const int mm = threadIdx.x;
        if (mm < kRows) {
            for (int j = 0; j < nt; ++j) {
                const float v = smem[kOffTileBestV + j * kRows + mm];
                const int i = reinterpret_cast<const int*>(smem)[kOffTileBestI + j * kRows + mm];
                if (better(v, i, run_v, run_i)) { run_v = v; run_i = i; }
            }
        }
    }
};

// ---------------------------------------------------------------- stages
// Embedding rows -> residual stream, first norm input, sums of squares.
template <class DT>
__device__ __forceinline__ void stage_embed(const DevModel& M, const float* __restrict__ gain, const PassArgs& P, int wg,
                                            int nwg) {
    const int k = P.k;
    const int ntiles = M.d / 16;
    // counts of the stages that split a tile over two workgroups: each returns to 0 by itself; a pass still starts clean
    if (wg == 0 && M.split_down)
        for (int i = threadIdx.x; i < kSplitTickets; i += kThreads)
            __hip_atomic_store(M.xch_ticket + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // 128 items per tile (16 rows x 8 column pairs); 4 tiles per sweep of the 512 threads
    const int sub = threadIdx.x >> 7, mm = (threadIdx.x >> 3) & 15, r = threadIdx.x & 7;
    for (int t0 = wg * 4; t0 < ntiles; t0 += nwg * 4) {
        const int tile = t0 + sub;
        const bool valid = tile < ntiles;
        float x1 = 0.f, x2 = 0.f;
        if (valid && mm < k) {
            const size_t o = (size_t)P.tokens[mm] * M.d + tile * 16 + r;
            if constexpr (DT::HAS_LO) {
                x1 = bf16_to_f32(reinterpret_cast<const uint16_t*>(M.embed)[o]);
                x2 = bf16_to_f32(reinterpret_cast<const uint16_t*>(M.embed)[o + 8]);
            } else {
                x1 = reinterpret_cast<const float*>(M.embed)[o];
                x2 = reinterpret_cast<const float*>(M.embed)[o + 8];
            }
        }
        float g1 = 0.f, g2 = 0.f;
        if (valid) { g1 = gain[tile * 16 + r]; g2 = gain[tile * 16 + r + 8]; }
        residual_pair<DT>(M, g1, g2, valid ? tile : 0, mm, r, x1, x2, k, valid && mm < k);
    }
}

// Cache rows of the kv heads whose attention units run on this workgroup's XCD, fetched into that XCD's L2 for
// the attention stage, which is next and waits on exactly those loads (the units of kv head h run on XCD h mod
// 8, and so does every workgroup with that index mod 8).  The calling workgroup is the rank-th of `count`
// workgroups of its XCD that share the job.  Only whole key blocks below the first position this pass writes are
// touched (one word per 128-byte line, delivered to LDS words nobody reads), so no line is fetched that this
// kernel may still change; and only as long as those rows are a small part of an XCD's L2 (they are read once;
// the O-projection's weights, fetched by the attention stage, need the rest of it).
template <class DT>
__device__ __forceinline__ void prefetch_cache_rows(const DevModel& M, const DevLayer& Ly, const PassArgs& P, int wg, int rank,
                                                    int count, float* smem) {
    const size_t per_xcd = (size_t)(M.Hkv >> 3) * 2 * P.L0 * M.hd * DT::ESZ;
    if (!kKvPrefetch || (M.Hkv & 7) != 0 || per_xcd > kKvPrefetchMax) return;
    const int x = wg & 7;
    const int safe = P.L0 / DT::BLOCK_KEYS * DT::BLOCK_KEYS;  // positions in blocks this pass leaves alone
    const int half = (int)((size_t)safe * M.hd * DT::ESZ / 128);   // lines of one head's keys (values alike)
    const int total = (M.Hkv >> 3) * 2 * half;                // lines for this XCD's kv heads
    const int share = (total + count - 1) / count;
    const size_t head_bytes = (size_t)M.ctx_pad * M.hd * DT::ESZ;
    const size_t slot_bytes = (size_t)P.slot0 * M.Hkv * head_bytes;
    const int end = (rank + 1) * share < total ? (rank + 1) * share : total;
    for (int line = rank * share + (int)threadIdx.x; line < end; line += kThreads) {
        const int hi = line / (2 * half), within = line % (2 * half);
        const char* base = reinterpret_cast<const char*>(within < half ? Ly.kcache : Ly.vcache);
        const char* p = base + slot_bytes + (size_t)(x + 8 * hi) * head_bytes +
                        (size_t)(within < half ? within : within - half) * 128;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                         (__attribute__((address_space(3))) void*)(smem + kOffPfSink + (threadIdx.x >> 6) * 64),
                                         4, 0, 0);
    }
    prefetch_retire();
}

template <class DT, bool ONE>
__device__ __forceinline__ void stage_qkv(const DevModel& M, const DevLayer& Ly, const PassArgs& P, int wg, int nwg,
                                          float* smem) {
    // All kernel arguments the stage needs in one batch at entry.  Left alone the compiler loads an argument where it
    // is first used, and the stage waited for argument memory six times in a row before its first weight load.
    pin_scalar(Ly.wqkv); pin_scalar(M.A); pin_scalar(M.ssq); pin_scalar(M.d); pin_scalar(M.nqkv); pin_scalar(P.k);
    pin_scalar(M.hd); pin_scalar(M.qdim); pin_scalar(M.kvdim); pin_scalar(M.Hkv); pin_scalar(M.ctx_pad);
    pin_scalar(M.rope_cos); pin_scalar(M.rope_sin); pin_scalar(M.Q_hi); pin_scalar(M.Q_lo); pin_scalar(M.eps);
    pin_scalar(Ly.kcache); pin_scalar(Ly.vcache); pin_scalar(P.L0); pin_scalar(P.slot0); pin_scalar(nwg);
    EpiQKV<DT, ONE> epi{M, Ly, smem + kOffRstd, P, P.k, {}, {}, {}, 0, 0};
    epi.begin();
    const int n_tiles = M.nqkv / 16;
    gemm_stage<DT>(Ly.wqkv, n_tiles, M.d / DT::KB, M.A, P.k, wg, nwg, epi, smem);
    // The workgroups that own one tile fewer than the others finish early and fetch cache rows meanwhile.
    if constexpr (ONE) {
        const int rounds = (n_tiles + nwg - 1) / nwg;
        const int w0 = n_tiles - (rounds - 1) * nwg;              // first workgroup with one tile fewer
        if (rounds > 1 && w0 < nwg && wg >= w0) {
            const int first = w0 + (((wg & 7) - w0) & 7);            // first such workgroup of this XCD
            prefetch_cache_rows<DT>(M, Ly, P, wg, (wg - first) >> 3, (nwg - first + 7) >> 3, smem);
        }
    }
}

template <class DT>
__device__ __forceinline__ void stage_oproj(const DevModel& M, const DevLayer& Ly, const PassArgs& P, int wg, int nwg,
                                            float* smem) {
    pin_scalar(Ly.wo); pin_scalar(M.O); pin_scalar(M.d); pin_scalar(M.qdim); pin_scalar(P.k);   // one batch, as in stage_qkv
    pin_scalar(M.X); pin_scalar(M.A); pin_scalar(M.ssq); pin_scalar(Ly.g_mlp); pin_scalar(nwg);
    EpiResidual<DT, 4> epi{M, Ly.g_mlp, P.k, {}, {}, {}, {}};
    gemm_stage<DT>(Ly.wo, M.d / 16, M.qdim / DT::KB, M.O, P.k, wg, nwg, epi, smem);
}

template <class DT>
__device__ __forceinline__ void stage_gateup(const DevModel& M, const DevLayer& Ly, const PassArgs& P, int wg, int nwg,
                                             float* smem) {
    pin_scalar(Ly.wgu); pin_scalar(M.A); pin_scalar(M.ssq); pin_scalar(M.d); pin_scalar(M.F); pin_scalar(P.k);   // one batch
    pin_scalar(M.H); pin_scalar(M.eps); pin_scalar(nwg);
    EpiSwiGLU<DT> epi{M, smem + kOffRstd, P.k, {}};
    epi.pre.begin(M, P.k);
    gemm_stage<DT>(Ly.wgu, 2 * M.F / 16, M.d / DT::KB, M.A, P.k, wg, nwg, epi, smem);
}

template <class DT>
__device__ __forceinline__ void stage_down(const DevModel& M, const DevLayer& Ly, const float* gain_next,
                                           const PassArgs& P, int wg, int nwg, float* smem) {
    pin_scalar(Ly.wd); pin_scalar(M.H); pin_scalar(M.d); pin_scalar(M.F); pin_scalar(P.k); pin_scalar(M.split_down);   // one batch
    pin_scalar(M.xch); pin_scalar(M.xch_ticket); pin_scalar(M.X); pin_scalar(M.A); pin_scalar(M.ssq); pin_scalar(gain_next); pin_scalar(nwg);
    EpiResidual<DT, 6> epi{M, gain_next, P.k, {}, {}, {}, {}};
    if (M.split_down == 1) gemm_stage_split<DT, 1, 2>(Ly.wd, M.d / 16, M.F / DT::KB, M.H, P.k, wg, epi, smem, M.xch, M.xch_ticket);
    else if (M.split_down == 2) gemm_stage_split<DT, 2, 2>(Ly.wd, M.d / 16, M.F / DT::KB, M.H, P.k, wg, epi, smem, M.xch, M.xch_ticket);
    else gemm_stage<DT>(Ly.wd, M.d / 16, M.F / DT::KB, M.H, P.k, wg, nwg, epi, smem);
}

template <class DT>
__device__ __forceinline__ void stage_lmhead(const DevModel& M, const PassArgs& P, int wg, int nwg, float* smem) {
    pin_scalar(M.wlm); pin_scalar(M.A); pin_scalar(M.ssq); pin_scalar(M.d); pin_scalar(M.V); pin_scalar(P.k);   // one batch
    pin_scalar(M.eps); pin_scalar(P.keep_logits); pin_scalar(M.logits); pin_scalar(M.lm_wgs); pin_scalar(M.best_val); pin_scalar(M.best_idx); pin_scalar(nwg);
    EpiLMHead epi{M, smem, P.k, P.keep_logits, -INFINITY, 0x7fffffff, {}};
    epi.pre.begin(M, P.k);
    gemm_stage<DT>(M.wlm, M.V / 16, M.d / DT::KB, M.A, P.k, wg, nwg, epi, smem);
    if (threadIdx.x < kRows && wg < M.lm_wgs) {
        M.best_val[wg * kRows + threadIdx.x] = epi.run_v;
        M.best_idx[wg * kRows + threadIdx.x] = epi.run_i;
    }
}

// Causal grouped-query attention: every sequence of the pass has its k rows
// checked against keys 0 .. L+k-1 of its own cache.
// Work unit = (sequence, kv head, chunk of 8 key blocks; a block is 32 keys bf16 / 16 keys
// fp32); tile rows of other sequences are masked out of the unit.  Wave w of the workgroup serves query head w % G of the group and the
// w / G -th run of G consecutive blocks, walking them in order with a running
// softmax (max, denominator, numerator) in registers; the next block's K and V
// fragments are fetched while the current one is used.  Scores are computed
// transposed (keys x rows) so that the matrix-core result registers are, after
// the softmax numerator, already the operand of the P.V product: nothing is
// transposed through LDS.  The 8/G runs of a head are merged through LDS in run
// order.  Block, run and chunk boundaries sit at fixed absolute positions, so a
// row's result does not depend on how many rows the pass has or where it starts.
// Output per (unit, head, row): numerator[hd], running max, denominator.
constexpr int kPartRow = 4;   // floats appended to a partial's numerator: max, denominator, 2 pad (keeps 16-byte alignment)

template <class DT, int HD, bool ONE>
__device__ __forceinline__ void stage_attention(const DevModel& M, const DevLayer& Ly, const PassArgs& P, int wg, int nwg,
                                                float* smem) {
    pin_scalar(M.Q_hi); pin_scalar(M.Q_lo); pin_scalar(Ly.kcache); pin_scalar(Ly.vcache); pin_scalar(M.att_part);
    pin_scalar(Ly.wo); pin_scalar(M.d); pin_scalar(M.qdim); pin_scalar(M.Hkv); pin_scalar(M.ctx_pad);
    pin_scalar(M.att_scale); pin_scalar(M.G); pin_scalar(M.bpw); pin_scalar(P.L0); pin_scalar(P.k);
    pin_scalar(P.nchunks0); pin_scalar(P.slot0); pin_scalar(P.units); pin_scalar(P.n_seg); pin_scalar(nwg);
    constexpr int FR = HD / 4 / DT::EPL;     // 16-byte fragments per lane along head_dim
    constexpr int HT = HD / 16;              // 16-wide head_dim tiles
    constexpr int BK = DT::BLOCK_KEYS, TPB = DT::TPB;
    constexpr int HDP = HD + kAttPad;
    const int last = P.n_seg - 1;
    const int units = P.units;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int G = M.G, bpw = M.bpw;
    const int lg = __builtin_ctz((unsigned)G);         // G is 1, 2, 4 or 8 (checked at model creation): shifts, no divisions
    const int parts = kWaves >> lg, hq = wave & (G - 1), part = wave >> lg;
    float* partO = smem;                               // [hq][part][16][HD + pad]
    float* partML = smem + kWaves * kRows * HDP;       // [hq][part][16][2]
    const int nblk = M.ctx_pad / BK;
    const uint4 zero4 = uint4{0, 0, 0, 0};
    // The O-projection's weights, fetched into L2 while this stage waits on latency, by the workgroups that have
    // no attention unit (at short contexts there are fewer units than compute units).  Such a workgroup serves the
    // O-projection workgroups of its own XCD in turn with the other idle workgroups of that XCD.
    if (kAttPf > 0 && wg >= units) {
        const NextWeights wo{Ly.wo, M.d / 16, M.qdim / DT::KB, true, EpiResidual<DT, 4>::kRotWg, EpiResidual<DT, 4>::kRotWave,
                              EpiResidual<DT, 4>::kInterleave, EpiResidual<DT, 4>::kOldShare};
        const int consumers = wo.n_tiles < nwg ? wo.n_tiles : nwg;      // workgroups of the O-projection
        const int x = wg & 7;
        const int first = units + ((x - units) & 7);                    // first idle workgroup of XCD x
        const int rank = (wg - first) >> 3, idle = (nwg - first + 7) >> 3;
        if (kAttPfSleep > 0) __builtin_amdgcn_s_sleep(kAttPfSleep);   // the units' own loads go first
        for (int t = rank, n = 0; x + 8 * t < consumers && n < kAttPfMax; t += idle, ++n)
            prefetch_frags<0, kAttPf>(wo, x + 8 * t, consumers, wave, lane, smem + kOffPfSink + wave * 64);
        prefetch_retire();
        return;
    }
    for (int u = wg; u < units; u += nwg) {
        int L = P.L0, k = P.k, row0 = 0, nchunks = P.nchunks0, cslot = P.slot0, unit0 = 0;
        if constexpr (!ONE) {
            int si = 0;
            while (si < last && u >= P.seg[si + 1].unit0) ++si;
            const PassSeg& S = P.seg[si];
            L = S.L; k = S.k; row0 = S.row0; nchunks = S.nchunks; cslot = S.slot; unit0 = S.unit0;
        }
        const int T = L + k;
        const int ul = u - unit0;
        // Which (kv head, chunk) this unit is.  With a multiple of 8 kv heads, all chunks of a kv head go to
        // workgroups of one XCD (workgroup index mod 8 = kv head mod 8), and so do the merge waves of its query
        // heads: they then find the chunk partials in their own L2 instead of behind another XCD's write-back.
        int kvh, c;
        if (M.Hkv == 8) {                                // the usual case, without the divisions
            kvh = ul & 7;
            c = ul >> 3;
        } else if ((M.Hkv & 7) == 0) {
            asm volatile("");   // a real branch: no speculative divisions for the case above
            const int b = ul >> 3;
            kvh = (ul & 7) + 8 * (b / nchunks);
            c = b % nchunks;
        } else {
            asm volatile("");
            kvh = ul / nchunks;
            c = ul % nchunks;
        }
        const int ucanon = unit0 + kvh * nchunks + c;      // where the merge stage looks for this unit's partials
        const size_t slot_frags = (size_t)cslot * M.Hkv * M.ctx_pad * HD / DT::EPL;   // 16-byte fragments per cache
        const bool mine = m >= row0 && m < row0 + k;     // tile row m belongs to this sequence
        const int head = kvh * G + hq;
        const int b0 = (c * parts + part) * bpw;       // first block of this wave's run
        uint4 qh[FR], ql[FR];
        {
            const int mq = mine ? m : row0;            // other rows mirror row0; fully masked, never written out
            const size_t q0 = (size_t)mq * M.qdim + head * HD + g * (HD / 4);
#pragma unroll
            for (int i = 0; i < FR; ++i) {
                qh[i] = load_frag<DT>(M.Q_hi, q0 + i * DT::EPL);
                ql[i] = zero4;
                if constexpr (DT::HAS_LO) ql[i] = load_frag<DT>(M.Q_lo, q0 + i * DT::EPL);
            }
        }
        uint4 kf[TPB][FR], vf[HT];
        auto load_block = [&](int b, uint4 (&kd)[TPB][FR], uint4 (&vd)[HT]) {
            const int bb = b < nblk ? b : nblk - 1;    // stay inside the cache allocation
            const uint4* kb = reinterpret_cast<const uint4*>(Ly.kcache) + slot_frags +
                              ((size_t)kvh * (M.ctx_pad / 16) + (size_t)bb * TPB) * FR * 64 + lane;
#pragma unroll
            for (int t = 0; t < TPB; ++t)
#pragma unroll
                for (int i = 0; i < FR; ++i) kd[t][i] = kb[(t * FR + i) * 64];
            const uint4* vb = reinterpret_cast<const uint4*>(Ly.vcache) + slot_frags +
                              (((size_t)kvh * nblk + bb) * HT) * 64 + lane;
#pragma unroll
            for (int j = 0; j < HT; ++j) vd[j] = vb[j * 64];
        };
        load_block(b0, kf, vf);
        float mrun = -INFINITY, lrun = 0.f;
        v4f o[HT];
#pragma unroll
        for (int j = 0; j < HT; ++j) o[j] = v4f{0.f, 0.f, 0.f, 0.f};
        for (int ib = 0; ib < bpw; ++ib) {
            const int p0 = (b0 + ib) * BK;
            if (p0 >= T) break;                         // wave-uniform: later blocks of the run hold no visible key
            uint4 kn[TPB][FR], vn[HT];
            // next block of the run, fetched while this one is used; at the run's last useful block, that block
            // again (a cache hit) rather than a block the neighbouring run owns: the fetch stays unconditional, so
            // it is issued ahead of the matrix instructions, but nothing waits for the last one before the end
            const bool more = ib + 1 < bpw && p0 + BK < T;
            load_block(more ? b0 + ib + 1 : b0 + ib, kn, vn);
            float sv[TPB][4];
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < TPB; ++t) {
                v4f sc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < FR; ++i) {
                    sc = DT::mfma_att(kf[t][i], qh[i], sc);
                    if constexpr (DT::HAS_LO) sc = DT::mfma_att(kf[t][i], ql[i], sc);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = p0 + t * 16 + g * 4 + e;
                    // causal: the sequence's j-th row (tile row row0+j) sees keys 0..L+j
                    sv[t][e] = mine && key <= L + m - row0 ? sc[e] * M.att_scale : -INFINITY;
                    mx = fmaxf(mx, sv[t][e]);
                }
            }
            mx = fmaxf(mx, lane_xor<16>(mx));
            mx = fmaxf(mx, lane_xor<32>(mx));
            const float mnew = fmaxf(mrun, mx);
            const float mref = mnew == -INFINITY ? 0.f : mnew;
            const float alpha = __expf(mrun - mref);     // 0 for the first visible block
            float pv[TPB][4], lsum = 0.f;
#pragma unroll
            for (int t = 0; t < TPB; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pv[t][e] = __expf(sv[t][e] - mref);
                    lsum += pv[t][e];
                }
            lsum = wave_xor_add<16>(lsum);
            lsum = wave_xor_add<32>(lsum);
            lrun = lrun * alpha + lsum;
            mrun = mnew;
            uint4 ph, pl = zero4;
            if constexpr (DT::HAS_LO) {
                uint32_t h[8], l[8];
#pragma unroll
                for (int t = 0; t < TPB; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        h[t * 4 + e] = DT::att_bits(pv[t][e]);
                        l[t * 4 + e] = DT::att_bits(pv[t][e] - DT::att_float(h[t * 4 + e]));
                    }
                ph = uint4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                pl = uint4{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
            } else {
                ph = uint4{__float_as_uint(pv[0][0]), __float_as_uint(pv[0][1]), __float_as_uint(pv[0][2]), __float_as_uint(pv[0][3])};
            }
#pragma unroll
            for (int j = 0; j < HT; ++j) {
                o[j] = o[j] * alpha;
                o[j] = DT::mfma_att(vf[j], ph, o[j]);
                if constexpr (DT::HAS_LO) o[j] = DT::mfma_att(vf[j], pl, o[j]);
            }
            if (!more) break;     // wave-uniform; the look-ahead fetch is retired at the end of the stage
#pragma unroll
            for (int t = 0; t < TPB; ++t)
#pragma unroll
                for (int i = 0; i < FR; ++i) kf[t][i] = kn[t][i];
#pragma unroll
            for (int j = 0; j < HT; ++j) vf[j] = vn[j];
        }
        // run partial to LDS: o[j][e] is head_dim index 16j + 4g + e of row m
        const int slot = hq * parts + part;
#pragma unroll
        for (int j = 0; j < HT; ++j)
            *reinterpret_cast<v4f*>(partO + ((size_t)(slot * kRows + m) * HDP + j * 16 + g * 4)) = o[j];
        if (g == 0) {
            partML[(slot * kRows + m) * 2 + 0] = mrun;
            partML[(slot * kRows + m) * 2 + 1] = lrun;
        }
        __syncthreads();
        // merge the runs of each head in run order; item = (head, row, 4 consecutive head_dim entries)
        for (int x = tid; x < G * kRows * (HD / 4); x += kThreads) {
            const int c4 = x % (HD / 4), mm = (x / (HD / 4)) % kRows, hh = x / (kRows * (HD / 4));
            if (mm < row0 || mm >= row0 + k) continue;
            float Mx = -INFINITY;
            for (int pp = 0; pp < parts; ++pp) Mx = fmaxf(Mx, partML[((hh * parts + pp) * kRows + mm) * 2]);
            float den = 0.f;
            v4f num = v4f{0.f, 0.f, 0.f, 0.f};
            for (int pp = 0; pp < parts; ++pp) {
                const int sl = hh * parts + pp;
                const float mw = partML[(sl * kRows + mm) * 2];
                const float wt = mw == -INFINITY ? 0.f : __expf(mw - Mx);
                den += wt * partML[(sl * kRows + mm) * 2 + 1];
                num += wt * *reinterpret_cast<const v4f*>(partO + ((size_t)(sl * kRows + mm) * HDP + c4 * 4));
            }
            float* out = M.att_part + (((size_t)ucanon * G + hh) * kRows + mm) * (HD + kPartRow);
            *reinterpret_cast<v4f*>(out + c4 * 4) = num;
            if (c4 == 0) { out[HD] = Mx; out[HD + 1] = den; }
        }
        __syncthreads();
    }
    prefetch_retire();
}

// Merge of the chunk partials of each (head, row) in chunk order -> normalised
// attention output as the O-projection's input.  One wave per (head, row):
// lanes first hold one chunk each (max, weight, denominator), then one slice of
// head_dim each.
template <class DT, int HD, bool ONE>
__device__ __forceinline__ void stage_attn_merge(const DevModel& M, const PassArgs& P, int wg, int nwg) {
    pin_scalar(M.att_part); pin_scalar(M.O); pin_scalar(M.Hq); pin_scalar(M.Hkv); pin_scalar(M.G); pin_scalar(M.chunk);
    pin_scalar(P.k); pin_scalar(P.L0); pin_scalar(P.nchunks0);
    (void)nwg;
    const int k = P.k, CS = M.chunk;
    const int lane = threadIdx.x & 63;
    // launched with one wave per workgroup and one workgroup per (head, row): no loop, so that what only the
    // rarer index forms below need (reciprocals for their divisions) is not computed ahead of it for all of them
    constexpr int PER = HD / 64, ROW = HD + kPartRow;
    const int x = wg;
    if (x < M.Hq * k) {
        int kvh, hq, mm;        // wave x -> (query head, row); same XCD as the attention units of the kv head
        if (M.Hkv == 8) {       // the usual case without divisions: x = 8 (hq k + mm) + kvh, hq < G <= 8
            const int y = x >> 3;
            kvh = x & 7;
            hq = (y >= k) + (y >= 2 * k) + (y >= 3 * k) + (y >= 4 * k) + (y >= 5 * k) + (y >= 6 * k) + (y >= 7 * k);
            mm = y - hq * k;
        } else if ((M.Hkv & 7) == 0) {
            asm volatile("");   // a real branch: the divisions below are not to be computed speculatively for the case above
            const int y = x >> 3, per = M.G * k;
            kvh = (x & 7) + 8 * (y / per);
            hq = (y % per) / k;
            mm = y % k;
        } else {
            asm volatile("");
            kvh = (x / k) / M.G;
            hq = (x / k) % M.G;
            mm = x % k;
        }
        const int head = kvh * M.G + hq;
        int unit0 = 0, nchunks = P.nchunks0, pos = P.L0 + mm;
        if constexpr (!ONE) {
            const PassSeg& S = P.seg[P.row_seg[mm]];
            unit0 = S.unit0;
            nchunks = S.nchunks;
            pos = P.row_pos[mm];
        }
        // chunks holding keys this row can see: pos / CS + 1.  For a pass of one sequence without the division: its
        // last row's count is nchunks, and a chunk has at least 16 keys, so the rows of a pass lie in at most two chunks
        int nch;
        if constexpr (ONE) nch = pos >= (nchunks - 1) * CS ? nchunks : nchunks - 1;
        else nch = pos / CS + 1;
        const float* base = M.att_part + ((((size_t)unit0 + (size_t)kvh * nchunks) * M.G + hq) * kRows + mm) * ROW;
        const size_t cstride = (size_t)M.G * kRows * ROW;
        float Mrun = -INFINITY, den = 0.f, num[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) num[i] = 0.f;
        // numerators of the first chunks are fetched together with the maxima: one memory round trip
        constexpr int CPRE = 24;
        float pre[CPRE][PER];
#pragma unroll
        for (int j = 0; j < CPRE; ++j) {
            const float* pj = base + (size_t)(j < nch ? j : nch - 1) * cstride;
#pragma unroll
            for (int i = 0; i < PER; ++i) pre[j][i] = pj[lane + 64 * i];
        }
        for (int c0 = 0; c0 < nch; c0 += 64) {        // groups of 64 chunks, in order
            const int cc = c0 + lane;
            const bool on = cc < nch;
            const float* p = base + (size_t)(on ? cc : c0) * cstride;
            const float mc = on ? p[HD] : -INFINITY;
            const float dc = on ? p[HD + 1] : 0.f;
            float Mg = mc;
            Mg = wave_max_all(Mg);
            const float Mnew = fmaxf(Mrun, Mg);       // finite: chunk 0 always holds key 0
            const float scale_old = __expf(Mrun - Mnew);
            const float wt = mc == -INFINITY ? 0.f : __expf(mc - Mnew);
            float dsum = wt * dc;
            dsum = wave_sum_all(dsum);
            den = den * scale_old + dsum;
#pragma unroll
            for (int i = 0; i < PER; ++i) num[i] *= scale_old;
            const int ng = nch - c0 < 64 ? nch - c0 : 64;
            if (c0 == 0) {
#pragma unroll
                for (int j = 0; j < CPRE; ++j) {
                    const float wj = j < ng ? lane_value(wt, j) : 0.f;
#pragma unroll
                    for (int i = 0; i < PER; ++i) num[i] += wj * pre[j][i];
                }
            }
            for (int j = c0 == 0 ? CPRE : 0; j < ng; ++j) {
                const float wj = lane_value(wt, j);
                const float* pj = base + (size_t)(c0 + j) * cstride;
#pragma unroll
                for (int i = 0; i < PER; ++i) num[i] += wj * pj[lane + 64 * i];
            }
            Mrun = Mnew;
        }
        const float inv = 1.0f / den;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            store_gemm_in<DT>(M.O, k, mm, head * HD + lane + 64 * i, num[i] * inv);
    }
}

// Arg-max across workgroups by wave shuffles (wave r reduces row r), then the
// mismatch test of Algorithm 1 on wave 0, per sequence: target = [p_ctx, g[0], .., g[k-2]]
// over the sequence's rows, accept the longest prefix with draft == target, emit the
// model's own token at the first mismatch (or g[k-1] when all match).  One workgroup of 16 waves.
__device__ __forceinline__ void stage_accept(const DevModel& M, const PassArgs& P, int* sg) {
    const int lane = threadIdx.x & 63, row = threadIdx.x >> 6;
    const int k = P.k;
    {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        if (row < k)
            for (int w = lane; w < M.lm_wgs; w += 64) {
                const float v = M.best_val[w * kRows + row];
                const int i = M.best_idx[w * kRows + row];
                if (better(v, i, bv, bi)) { bv = v; bi = i; }
            }
        keep_better_xor<32>(bv, bi);
        keep_better_xor<16>(bv, bi);
        keep_better_xor<8>(bv, bi);
        keep_better_xor<4>(bv, bi);
        keep_better_xor<2>(bv, bi);
        keep_better_xor<1>(bv, bi);
        if (lane == 0) sg[row] = row < k ? bi : -1;
    }
    __syncthreads();
    if (row != 0) return;
    const int myg = lane < kRows ? sg[lane] : -1;
    if (lane < kRows) M.res->greedy[lane] = myg;
    // lane r holds g[r]; for the sequence's first row the target is its p_ctx, else the previous row's g
    const int rl = lane < kRows ? lane : 0;
    const PassSeg& Sr = P.seg[P.row_seg[rl]];
    const int prev = __shfl_up(myg, 1, 64);
    const int target = rl == Sr.row0 ? Sr.p_ctx : prev;
    const bool match = lane < k && (P.force_accept || P.tokens[rl] == target);
    const unsigned long long ball = __ballot(match);
    // lane s now serves segment s
    const int sl = lane < P.n_seg ? lane : 0;
    const PassSeg& S = P.seg[sl];
    const unsigned long long seg_match = (ball >> S.row0) & ((1ull << S.k) - 1ull);
    const int n = __ffsll((long long)~seg_match) - 1;                       // first row of the segment that does not match; k if none
    const int gk = __shfl(myg, S.row0 + S.k - 1, 64);
    const int nxt_t = __shfl(target, S.row0 + (n < S.k ? n : 0), 64);
    if (lane < P.n_seg) {
        M.res->accept_len[lane] = n;
        M.res->next_token[lane] = n < S.k ? nxt_t : gk;
    }
}

// ---------------------------------------------------------------- one kernel per stage
#define AMUSD_STAGE_KERNEL(name, body)                                                                     \
    template <class DT, int HD, bool ONE = false>                                                            \
    __global__ void __launch_bounds__(kThreads) name(DevModel M, DevLayer Ly, const float* gain, PassArgs P) { \
        extern __shared__ float smem[];                                                                      \
        (void)smem; (void)gain; (void)Ly;                                                                    \
        body;                                                                                                \
    }

AMUSD_STAGE_KERNEL(k_embed, (stage_embed<DT>(M, gain, P, blockIdx.x, gridDim.x)))
AMUSD_STAGE_KERNEL(k_qkv, (stage_qkv<DT, ONE>(M, Ly, P, blockIdx.x, gridDim.x, smem)))
AMUSD_STAGE_KERNEL(k_attention, (stage_attention<DT, HD, ONE>(M, Ly, P, blockIdx.x, gridDim.x, smem)))
AMUSD_STAGE_KERNEL(k_attn_merge, (stage_attn_merge<DT, HD, ONE>(M, P, blockIdx.x, gridDim.x)))
AMUSD_STAGE_KERNEL(k_oproj, (stage_oproj<DT>(M, Ly, P, blockIdx.x, gridDim.x, smem)))
AMUSD_STAGE_KERNEL(k_gateup, (stage_gateup<DT>(M, Ly, P, blockIdx.x, gridDim.x, smem)))
AMUSD_STAGE_KERNEL(k_down, (stage_down<DT>(M, Ly, gain, P, blockIdx.x, gridDim.x, smem)))
AMUSD_STAGE_KERNEL(k_lmhead, (stage_lmhead<DT>(M, P, blockIdx.x, gridDim.x, smem)))

__global__ void __launch_bounds__(kRows * 64) k_accept(DevModel M, PassArgs P) {
    __shared__ int sg[kRows];
    stage_accept(M, P, sg);
}

// ---------------------------------------------------------------- weight re-layout (model load)
template <class DT>
__global__ void k_relayout(uint4* __restrict__ dst, const void* __restrict__ src, int K, int n_tiles, int tile_offset,
                           int kind, int hd) {
    const int kblocks = K / DT::KB;
    const size_t total = (size_t)n_tiles * kblocks * 64;
    for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(x & 63);
        const size_t f = x >> 6;
        const int kb = (int)(f % kblocks);
        const int t = (int)(f / kblocks);
        const int r = lane & 15, g = lane >> 4;
        long row;
        if (kind == kNatural) {
            row = (long)t * 16 + r;
        } else if (kind == kRopePairs) {
            const int tph = hd / 16;
            row = (long)(t / tph) * hd + (t % tph) * 8 + (r & 7) + (r >> 3) * (hd / 2);
        } else if (kind == kGate) {
            if (r >= 8) continue;
            row = (long)t * 8 + r;
        } else {
            if (r < 8) continue;
            row = (long)t * 8 + r - 8;
        }
        const uint4 v = load_frag<DT>(src, (size_t)row * K + (size_t)kb * DT::KB + g * DT::EPL);
        dst[((size_t)(tile_offset + t) * kblocks + kb) * 64 + lane] = v;
    }
}

hipError_t launch_relayout(int dtype, uint4* dst, const void* src, int K, int n_tiles, int tile_offset, int kind,
                           int hd, hipStream_t stream) {
    const int kb = dtype ? BF16::KB : FP32::KB;
    const size_t total = (size_t)n_tiles * (K / kb) * 64;
    const int grid = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    if (dtype)
        hipLaunchKernelGGL(k_relayout<BF16>, dim3(grid), dim3(256), 0, stream, dst, src, K, n_tiles, tile_offset, kind, hd);
    else
        hipLaunchKernelGGL(k_relayout<FP32>, dim3(grid), dim3(256), 0, stream, dst, src, K, n_tiles, tile_offset, kind, hd);
    return hipGetLastError();
}

// ---------------------------------------------------------------- plain copy (profiler calibration)
__global__ void __launch_bounds__(256) k_plain_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

hipError_t launch_copy(uint4* dst, const uint4* src, size_t n, hipStream_t stream) {
    hipLaunchKernelGGL(k_plain_copy, dim3(2048), dim3(256), 0, stream, dst, src, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------- zero fill (a kernel, so no memset node is needed)
__global__ void __launch_bounds__(256) k_fill_zero(uint4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = uint4{0, 0, 0, 0};
}

hipError_t launch_fill_zero(uint4* dst, size_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const size_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0, stream, dst, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------- bare streaming kernel (what a chain of dependent kernels can reach)
// Reads `iters` x 8 KiB per workgroup (one contiguous run per workgroup, 16 non-temporal 16-byte loads in flight per
// thread: the load pattern of the GEMM stages without their arithmetic), folds the data into one word per workgroup,
// and chains on the previous launch through a 256-float vector it reads and rewrites.
__global__ void __launch_bounds__(kThreads) k_stream_only(const uint4* __restrict__ src, int iters, const float* __restrict__ in,
                                                          float* __restrict__ out, unsigned* __restrict__ fold) {
    constexpr int PF = 16;
    const int tid = threadIdx.x, wg = blockIdx.x;
    const uint4* p = src + (size_t)wg * iters * kThreads + tid;
    const int last = iters - 1;
    uint4 buf[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) buf[i] = load_stream(p + (size_t)(i < last ? i : last) * kThreads);
    const float a = in[(wg + 1) & 255];
    unsigned acc = 0;
    int s0 = 0;
    for (; s0 + PF < iters; s0 += PF) {
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            acc += buf[i].x ^ buf[i].y ^ buf[i].z ^ buf[i].w;
            const int sn = s0 + i + PF < last ? s0 + i + PF : last;
            buf[i] = load_stream(p + (size_t)sn * kThreads);
        }
    }
#pragma unroll
    for (int i = 0; i < PF; ++i)
        if (s0 + i < iters) acc += buf[i].x ^ buf[i].y ^ buf[i].z ^ buf[i].w;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((tid & 63) == 0) atomicAdd(&fold[wg & 255], acc);
    if (tid == 0) out[wg & 255] = a + 1.0f;
}

hipError_t launch_stream_chain(const uint4* buf, size_t buf_words, size_t words_per_kernel, int n_kernels, float* io,
                               unsigned* fold, hipStream_t stream) {
    // words_per_kernel is a multiple of 256 workgroups x 512 threads; regions rotate through the buffer
    const int iters = (int)(words_per_kernel / ((size_t)256 * kThreads));
    const size_t regions = buf_words / words_per_kernel;
    for (int i = 0; i < n_kernels; ++i) {
        const uint4* src = buf + (size_t)(i % regions) * words_per_kernel;
        hipLaunchKernelGGL(k_stream_only, dim3(256), dim3(kThreads), 0, stream, src, iters, io + 256 * (i & 1),
                           io + 256 * ((i + 1) & 1), fold);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- pass launch
constexpr size_t kSmemBytes = (size_t)kSmemFloats * sizeof(float);

template <class DT, int HD>
static hipError_t configure_one() {
    hipError_t e;
#define AMUSD_SET(kern)                                                                                          \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kern<DT, HD>), hipFuncAttributeMaxDynamicSharedMemorySize, \
                            (int)kSmemBytes);                                                                     \
    if (e != hipSuccess) return e;
    AMUSD_SET(k_qkv)
    AMUSD_SET(k_attention)
#define AMUSD_SET_ONE(kern)                                                                                        \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kern<DT, HD, true>),                                     \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmemBytes);                           \
    if (e != hipSuccess) return e;
    AMUSD_SET_ONE(k_qkv)
    AMUSD_SET_ONE(k_attention)
#undef AMUSD_SET_ONE
    AMUSD_SET(k_oproj)
    AMUSD_SET(k_gateup)
    AMUSD_SET(k_down)
    AMUSD_SET(k_lmhead)
#undef AMUSD_SET
    return hipSuccess;
}


hipError_t configure_kernels() {
    hipError_t e;
    if ((e = configure_one<BF16, 64>()) != hipSuccess) return e;
    if ((e = configure_one<BF16, 128>()) != hipSuccess) return e;
    if ((e = configure_one<FP32, 64>()) != hipSuccess) return e;
    if ((e = configure_one<FP32, 128>()) != hipSuccess) return e;
    return hipSuccess;
}

template <class DT, int HD>
static hipError_t launch_pass_t(const DevModel& M, const DevLayer* Ls, const PassArgs& P, int nwg, hipStream_t s,
                                StageTimer* tm) {
    const dim3 blk(kThreads);
    const int embed_wgs = (M.d / 16 + 3) / 4 < nwg ? (M.d / 16 + 3) / 4 : nwg;
    const int att_units = P.units;
    const int att_wgs = kAttPf > 0 ? nwg : att_units < nwg ? att_units : nwg;   // idle ones fetch ahead
    const int merge_wgs = M.Hq * P.k;      // one wave each
    const int qkv_wgs = M.nqkv / 16 < nwg ? M.nqkv / 16 : nwg;
    const int d_wgs = M.d / 16 < nwg ? M.d / 16 : nwg;
    const int gu_wgs = 2 * M.F / 16 < nwg ? 2 * M.F / 16 : nwg;
    if (tm) tm->used = 0;
    // A timed stage is launched through the extended launch call, whose two events take the kernel's own
    // begin and end timestamps (no marker packets around it).
    const float* nogain = nullptr;
#define AMUSD_LAUNCH_T(stage_id, kern, grid, block, smem, layer, gain)                                          \
    if (tm && tm->stage == stage_id) {                                                                            \
        hipExtLaunchKernelGGL((kern<DT, HD>), dim3(grid), block, smem, s, tm->begin[tm->used], tm->end[tm->used], \
                              0, M, Ls[layer], gain, P);                                                        \
        ++tm->used;                                                                                              \
    } else {                                                                                                     \
        hipLaunchKernelGGL((kern<DT, HD>), dim3(grid), block, smem, s, M, Ls[layer], gain, P);                  \
    }
#define AMUSD_LAUNCH(stage_id, kern, grid, smem, layer, gain) AMUSD_LAUNCH_T(stage_id, kern, grid, blk, smem, layer, gain)
    // the stages that place rows in their sequences have a second form for a pass of one sequence
#define AMUSD_LAUNCH_SEQ(stage_id, kern, grid, block, smem, layer)                                                \
    if (P.n_seg == 1) {                                                                                           \
        if (tm && tm->stage == stage_id) {                                                                        \
            hipExtLaunchKernelGGL((kern<DT, HD, true>), dim3(grid), block, smem, s, tm->begin[tm->used],            \
                                  tm->end[tm->used], 0, M, Ls[layer], nogain, P);                                 \
            ++tm->used;                                                                                           \
        } else {                                                                                                  \
            hipLaunchKernelGGL((kern<DT, HD, true>), dim3(grid), block, smem, s, M, Ls[layer], nogain, P);          \
        }                                                                                                         \
    } else {                                                                                                      \
        AMUSD_LAUNCH_T(stage_id, kern, grid, block, smem, layer, nogain)                                          \
    }
    AMUSD_LAUNCH(0, k_embed, embed_wgs, 0, 0, Ls[0].g_attn)
    for (int l = 0; l < M.n_layers; ++l) {
        const float* gain_next = l + 1 < M.n_layers ? Ls[l + 1].g_attn : M.g_final;
        AMUSD_LAUNCH_SEQ(1, k_qkv, qkv_wgs, blk, kSmemBytes, l)
        AMUSD_LAUNCH_SEQ(2, k_attention, att_wgs, blk, kSmemBytes, l)
        AMUSD_LAUNCH_SEQ(3, k_attn_merge, merge_wgs, dim3(64), 0, l)
        AMUSD_LAUNCH(4, k_oproj, d_wgs, kSmemBytes, l, nogain)
        AMUSD_LAUNCH(5, k_gateup, gu_wgs, kSmemBytes, l, nogain)
        AMUSD_LAUNCH(6, k_down, (M.split_down == 1 ? 2 * d_wgs : d_wgs), kSmemBytes, l, gain_next)
    }
    AMUSD_LAUNCH(7, k_lmhead, M.lm_wgs, kSmemBytes, 0, nogain)
#undef AMUSD_LAUNCH_SEQ
#undef AMUSD_LAUNCH
#undef AMUSD_LAUNCH_T
    if (tm && tm->stage == 8) {
        hipExtLaunchKernelGGL(k_accept, dim3(1), dim3(kRows * 64), 0, s, tm->begin[0], tm->end[0], 0, M, P);
        tm->used = 1;
    } else {
        hipLaunchKernelGGL(k_accept, dim3(1), dim3(kRows * 64), 0, s, M, P);
    }
    return hipGetLastError();
}

hipError_t launch_pass(const DevModel& M, const DevLayer* Ls, const PassArgs& P, int nwg, hipStream_t stream,
                       StageTimer* tm) {
    if (M.dtype)
        return M.hd == 128 ? launch_pass_t<BF16, 128>(M, Ls, P, nwg, stream, tm)
                           : launch_pass_t<BF16, 64>(M, Ls, P, nwg, stream, tm);
    return M.hd == 128 ? launch_pass_t<FP32, 128>(M, Ls, P, nwg, stream, tm)
                       : launch_pass_t<FP32, 64>(M, Ls, P, nwg, stream, tm);
}

}  // namespace amusd
