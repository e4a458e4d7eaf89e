// Host side of the verify-pass library: the C ABI of include/amusd.h.
// Model set-up (allocation, weight re-layout), per-pass argument checks and
// launches, O(1) cache rollback, and the decoding loops of Algorithm 1.
#include "../../include/amusd.h"

#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "amusd_launch.h"
#include "amusd_loops.h"

using namespace amusd;

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string& msg) {
    g_last_error = msg;
    return code;
}

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess)                                                                           \
            return fail(AMUSD_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));                \
    } while (0)

struct HostStage {          // pinned: what one pass receives from the device
    PassResult res;
};

}  // namespace

// Workspace of the entry point that allocates nothing (amusd_verify_static): the buffers a pass keeps between its
// stages (residual stream, GEMM inputs, queries, attention partials, arg-max partials) laid out in this one array
// instead of the model's own allocations.  Every GPU the library runs on holds its own copy at its own address; in
// host code the array's name is only a stand-in, so the address is asked for once per device, with that device
// current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)AMUSD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};          // device address of `scratch`, per device
uint64_t g_scratch_owner[kMaxDevices] = {};     // model whose pass last laid out the array (0: none)
uint64_t g_next_model_id = 1;

// Device address of this device's copy of `scratch`; asked for on the first call per device.
hipError_t static_scratch_address(int device, void** out) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}
}  // namespace

struct SeqState {            // one sequence: its cache slot's length and the model's next token
    int kv_len = 0;
    int p_next = -1;
    std::vector<int> greedy_at;            // greedy_at[pos] = model's token for position pos, -1 unknown
};

struct SegReq {              // one sequence's share of a pass
    int seq;
    int L;
    const int32_t* tokens;
    int k;
};

struct amusd_model {
    amusd_config cfg{};
    hipStream_t stream = nullptr;
    int device = 0;
    int nwg = 0;
    bool finalized = false;
    bool keep_logits = false;
    bool logits_valid = false;
    int last_rows = 0;
    int n_seqs = 1;
    std::vector<SeqState> seqs;
    std::vector<char> have;                // tensors received
    std::vector<void*> allocs;             // everything to hipFree
    std::vector<DevLayer> layers_host;
    DevModel dm{};
    DevModel dm_static{};                  // dm with the pass workspace inside the static scratch array
    size_t static_bytes = 0;               // bytes of the array that workspace takes
    uint64_t id = 0;
    HostStage* hstage = nullptr;
    void* staging = nullptr;               // device staging for host-provided tensors
    size_t staging_bytes = 0;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    float last_ms = 0.f;
    StageTimer timer;
    std::vector<hipEvent_t> tev_begin, tev_end;
    double stage_ms = 0.0;
    int64_t stage_launches = 0;
    int64_t last_positions = 0;             // cache positions the last pass's attention read, all sequences
    int esz() const { return cfg.dtype == AMUSD_DTYPE_BF16 ? 2 : 4; }
    int kb() const { return cfg.dtype == AMUSD_DTYPE_BF16 ? 32 : 16; }
    int block_keys() const { return cfg.dtype == AMUSD_DTYPE_BF16 ? 32 : 16; }
};

namespace {

int dev_alloc(amusd_model* m, void** p, size_t bytes, bool zero) {
    HIP_TRY(hipMalloc(p, bytes ? bytes : 16));
    m->allocs.push_back(*p);
    if (zero) HIP_TRY(hipMemsetAsync(*p, 0, bytes ? bytes : 16, m->stream));
    return AMUSD_OK;
}

int check_config(const amusd_config* c) {
    if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 || c->vocab < 1 ||
        c->max_ctx < 1)
        return fail(AMUSD_E_ARG, "config: non-positive dimension");
    if (c->dtype != AMUSD_DTYPE_FP32 && c->dtype != AMUSD_DTYPE_BF16) return fail(AMUSD_E_ARG, "config: unknown dtype");
    if (c->max_k < 1 || c->max_k > AMUSD_MAX_K) return fail(AMUSD_E_ARG, "config: max_k outside [1,16]");
    if (c->max_seqs < 0 || c->max_seqs > AMUSD_MAX_SEQS) return fail(AMUSD_E_ARG, "config: max_seqs outside [0, AMUSD_MAX_SEQS]");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(AMUSD_E_ARG, "config: head_dim must be 64 or 128");
    if (c->n_q_heads % c->n_kv_heads) return fail(AMUSD_E_ARG, "config: n_q_heads not a multiple of n_kv_heads");
    {
        const int G = c->n_q_heads / c->n_kv_heads;
        if (G != 1 && G != 2 && G != 4 && G != 8)
            return fail(AMUSD_E_ARG, "config: n_q_heads / n_kv_heads must be 1, 2, 4 or 8");
    }
    const int kb = c->dtype == AMUSD_DTYPE_BF16 ? 32 : 16;
    const long qdim = (long)c->n_q_heads * c->head_dim;
    if (c->d_model % kb || qdim % kb || c->d_ffn % kb)
        return fail(AMUSD_E_ARG, "config: d_model, n_q_heads*head_dim and d_ffn must be multiples of the fragment width");
    if (c->d_model % 16 || c->d_ffn % 16 || c->vocab % 16)
        return fail(AMUSD_E_ARG, "config: d_model, d_ffn and vocab must be multiples of 16");
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return fail(AMUSD_E_ARG, "config: rope_theta/rms_eps");
    return AMUSD_OK;
}

struct TensorInfo {
    long rows, cols;
    bool per_layer;
};

TensorInfo tensor_info(const amusd_config& c, int id) {
    const long d = c.d_model, q = (long)c.n_q_heads * c.head_dim, kv = (long)c.n_kv_heads * c.head_dim, F = c.d_ffn,
               V = c.vocab;
    switch (id) {
        case AMUSD_T_EMBED: return {V, d, false};
        case AMUSD_T_LM_HEAD: return {V, d, false};
        case AMUSD_T_FINAL_NORM: return {1, d, false};
        case AMUSD_T_WQ: return {q, d, true};
        case AMUSD_T_WK: return {kv, d, true};
        case AMUSD_T_WV: return {kv, d, true};
        case AMUSD_T_WO: return {d, q, true};
        case AMUSD_T_WG: return {F, d, true};
        case AMUSD_T_WU: return {F, d, true};
        case AMUSD_T_WD: return {d, F, true};
        case AMUSD_T_NORM_ATTN: return {1, d, true};
        default: return {1, d, true};
    }
}

const char* kTensorNames[AMUSD_T_COUNT] = {"embed", "lm_head", "final_norm", "wq", "wk", "wv", "wo", "wg", "wu", "wd",
                                           "norm_attn", "norm_mlp"};

float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

float half_bits_to_float(uint16_t h) {      // IEEE binary16 -> float
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu, f = h & 0x3FFu, u;
    if (e == 0) {
        if (f == 0) {
            u = sign;
        } else {                             // subnormal: normalise
            int sh = 0;
            while (!(f & 0x400u)) { f <<= 1; ++sh; }
            u = sign | ((uint32_t)(113 - sh) << 23) | ((f & 0x3FFu) << 13);
        }
    } else if (e == 31) {
        u = sign | 0x7F800000u | (f << 13);
    } else {
        u = sign | ((e + 112) << 23) | (f << 13);
    }
    float r;
    std::memcpy(&r, &u, 4);
    return r;
}

std::once_flag g_cfg_once;
hipError_t g_cfg_err = hipSuccess;

// Runs one pass: segment i feeds segs[i].k tokens of sequence segs[i].seq at cache length segs[i].L.
// Everything is already validated (distinct sequences, lengths, capacity, tokens, row total).
int run_pass(amusd_model* m, const SegReq* segs, int n_seg, bool force_accept, bool use_static = false) {
    HostStage* h = m->hstage;
    if (use_static) {
        // The array keeps what the last call on this GPU left in it.  A pass reads only what it has written itself
        // in rows it owns, so nothing has to start at zero; the region is still cleared when another model used it
        // last, so that the unused rows of the 16-row tiles never hold another model's values.  A fill kernel, not a
        // memset: the call allocates nothing and stays usable where memset nodes are not.
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (g_scratch_owner[m->device] != m->id) {
            HIP_TRY(launch_fill_zero(reinterpret_cast<uint4*>(g_scratch_ptr[m->device]), m->static_bytes / 16, m->stream));
            g_scratch_owner[m->device] = m->id;
        }
    }
    const DevModel& D = use_static ? m->dm_static : m->dm;
    PassArgs P;
    std::memset(&P, 0, sizeof(P));
    int rows = 0, units = 0;
    int64_t positions = 0;
    for (int i = 0; i < n_seg; ++i) {
        const SegReq& r = segs[i];
        PassSeg& S = P.seg[i];
        S.L = r.L;
        S.k = r.k;
        S.row0 = rows;
        S.p_ctx = m->seqs[r.seq].greedy_at[r.L];
        S.slot = r.seq;
        S.unit0 = units;
        S.nchunks = (r.L + r.k + m->dm.chunk - 1) / m->dm.chunk;
        for (int j = 0; j < r.k; ++j) {
            P.tokens[rows + j] = r.tokens[j];
            P.row_pos[rows + j] = r.L + j;
            P.row_seg[rows + j] = i;
        }
        rows += r.k;
        units += m->dm.Hkv * S.nchunks;
        positions += r.L + r.k;
    }
    P.k = rows;
    P.n_seg = n_seg;
    P.L0 = P.seg[0].L;
    P.slot0 = P.seg[0].slot;
    P.nchunks0 = P.seg[0].nchunks;
    P.units = units;
    P.force_accept = force_accept ? 1 : 0;
    P.keep_logits = m->keep_logits ? 1 : 0;
    HIP_TRY(hipEventRecord(m->ev0, m->stream));
    HIP_TRY(launch_pass(D, m->layers_host.data(), P, m->nwg, m->stream, m->timer.stage >= 0 ? &m->timer : nullptr));
    HIP_TRY(hipEventRecord(m->ev1, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    HIP_TRY(hipEventElapsedTime(&m->last_ms, m->ev0, m->ev1));
    if (m->timer.stage >= 0) {
        for (int i = 0; i < m->timer.used; ++i) {
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, m->timer.begin[i], m->timer.end[i]));
            m->stage_ms += ms;
        }
        m->stage_launches += m->timer.used;
    }
    m->last_positions = positions;
    m->logits_valid = m->keep_logits;
    m->last_rows = rows;
    for (int i = 0; i < n_seg; ++i)
        if (h->res.accept_len[i] < 0 || h->res.accept_len[i] > segs[i].k)
            return fail(AMUSD_E_HIP, "pass returned an impossible accept_len");
    for (int i = 0; i < n_seg; ++i) {
        SeqState& q = m->seqs[segs[i].seq];
        for (int j = 0; j < segs[i].k; ++j) q.greedy_at[segs[i].L + j + 1] = h->res.greedy[P.seg[i].row0 + j];
        q.kv_len = segs[i].L + h->res.accept_len[i];
        q.p_next = h->res.next_token[i];
    }
    return AMUSD_OK;
}

int run_pass(amusd_model* m, int seq, int L, const int32_t* tokens, int k, bool force_accept) {
    const SegReq r{seq, L, tokens, k};
    return run_pass(m, &r, 1, force_accept);
}

int check_tokens(const amusd_model* m, const int32_t* t, int n) {
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= m->cfg.vocab) return fail(AMUSD_E_TOKEN, "token id outside [0, vocab)");
    return AMUSD_OK;
}

int need_ready(const amusd_model* m) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    if (!m->finalized) return fail(AMUSD_E_STATE, "model not finalized");
    return AMUSD_OK;
}

int need_seq(const amusd_model* m, int seq) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    if (seq < 0 || seq >= m->n_seqs) return fail(AMUSD_E_ARG, "sequence id outside [0, max_seqs)");
    return AMUSD_OK;
}

}  // namespace

extern "C" {

const char* amusd_strerror(int code) {
    switch (code) {
        case AMUSD_OK: return "ok";
        case AMUSD_E_ARG: return "invalid argument";
        case AMUSD_E_RANGE: return "length outside [0, kv_len]";
        case AMUSD_E_CAPACITY: return "key-value cache capacity exceeded";
        case AMUSD_E_TOKEN: return "token id outside the vocabulary";
        case AMUSD_E_STATE: return "model state does not allow the call";
        case AMUSD_E_HIP: return "HIP runtime error";
        case AMUSD_E_NOMEM: return "out of host memory";
        default: return "unknown error code";
    }
}

const char* amusd_last_error(void) { return g_last_error.c_str(); }

int amusd_model_create(const amusd_config* cfg, void* hip_stream, amusd_model** out) {
    if (!cfg || !out) return fail(AMUSD_E_ARG, "null argument");
    int rc = check_config(cfg);
    if (rc) return rc;
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (ndev < 1) return fail(AMUSD_E_HIP, "no HIP device");
    std::call_once(g_cfg_once, [] { g_cfg_err = configure_kernels(); });
    if (g_cfg_err != hipSuccess) return fail(AMUSD_E_HIP, std::string("configure_kernels: ") + hipGetErrorString(g_cfg_err));

    amusd_model* m = new (std::nothrow) amusd_model();
    if (!m) return fail(AMUSD_E_NOMEM, "model allocation");
    m->cfg = *cfg;
    m->stream = reinterpret_cast<hipStream_t>(hip_stream);
    auto bail = [&](int code) {
        amusd_model_free(m);
        return code;
    };
    if (hipGetDevice(&m->device) != hipSuccess) return bail(fail(AMUSD_E_HIP, "hipGetDevice"));
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, m->device) != hipSuccess) return bail(fail(AMUSD_E_HIP, "hipGetDeviceProperties"));
    m->nwg = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    const amusd_config& c = m->cfg;
    const int esz = m->esz(), BK = m->block_keys();
    DevModel& D = m->dm;
    D.n_layers = c.n_layers; D.d = c.d_model; D.Hq = c.n_q_heads; D.Hkv = c.n_kv_heads; D.hd = c.head_dim;
    D.F = c.d_ffn; D.V = c.vocab; D.G = c.n_q_heads / c.n_kv_heads;
    D.qdim = c.n_q_heads * c.head_dim; D.kvdim = c.n_kv_heads * c.head_dim; D.nqkv = D.qdim + 2 * D.kvdim;
    D.dtype = c.dtype;
    m->n_seqs = c.max_seqs > 0 ? c.max_seqs : 1;
    D.n_slots = m->n_seqs;
    {   // attention work units: about one per CU when the sequences of a pass (two, for a model that holds
        // several) are at full context, each wave walking bpw key blocks
        const int parts = kWaves / D.G;
        const int share = D.Hkv * (m->n_seqs > 1 ? 2 : 1);
        const int per_kvh = m->nwg / share > 0 ? m->nwg / share : 1;
        const long unit_min = (long)parts * BK;
        long bpw = (c.max_ctx + per_kvh * unit_min - 1) / (per_kvh * unit_min);
        if (bpw < 1) bpw = 1;
        D.bpw = (int)bpw;
        D.chunk = (int)(parts * bpw * BK);
    }
    D.max_ctx = c.max_ctx;
    D.ctx_pad = (c.max_ctx + D.chunk - 1) / D.chunk * D.chunk;
    D.max_chunks = D.ctx_pad / D.chunk;
    D.eps = c.rms_eps;
    D.att_scale = 1.0f / std::sqrt((float)c.head_dim);
    {   // Down projection: pairs of workgroups share K ranges when the contraction is long enough to pay for the
        // hand-over: a tile per pair (tiles for at most half the compute units: every compute unit gets work) or
        // two tiles per pair (a tile per compute unit: half the activation bytes per weight byte).  The same
        // scheme on the QKV projection (three tiles per pair at the 8B shape instead of two or one tile per
        // workgroup) measured no faster and is not built in.
        const int tiles = c.d_model / 16, kblocks = c.d_ffn / m->kb(), pairs = m->nwg / 2;
        const bool long_k = kblocks % 2 == 0 && kblocks / kWaves >= 16;
        D.split_down = !long_k || pairs > kSplitTickets ? 0 : 2 * tiles <= m->nwg ? 1 : tiles == m->nwg ? 2 : 0;
    }
    const int lm_tiles = c.vocab / 16;
    D.lm_wgs = lm_tiles < m->nwg ? lm_tiles : m->nwg;

    m->seqs.resize(m->n_seqs);
    for (SeqState& q : m->seqs) q.greedy_at.assign((size_t)c.max_ctx + kRows + 1, -1);
    m->have.assign((size_t)AMUSD_T_COUNT * (c.n_layers + 1), 0);
    m->layers_host.resize(c.n_layers);

    const size_t d = D.d, F = D.F, V = D.V, q = D.qdim;
    void* p = nullptr;
#define ALLOC(dst, type, bytes, zero)                          \
    if ((rc = dev_alloc(m, &p, (bytes), (zero))) != AMUSD_OK) return bail(rc); \
    dst = reinterpret_cast<type>(p);
    for (int l = 0; l < c.n_layers; ++l) {
        DevLayer& Ly = m->layers_host[l];
        ALLOC(Ly.wqkv, const uint4*, (size_t)D.nqkv * d * esz, false)
        ALLOC(Ly.wo, const uint4*, d * q * esz, false)
        ALLOC(Ly.wgu, const uint4*, 2 * F * d * esz, false)
        ALLOC(Ly.wd, const uint4*, d * F * esz, false)
        ALLOC(Ly.g_attn, const float*, d * 4, false)
        ALLOC(Ly.g_mlp, const float*, d * 4, false)
        ALLOC(Ly.kcache, void*, (size_t)D.n_slots * D.Hkv * D.ctx_pad * D.hd * esz, true)
        ALLOC(Ly.vcache, void*, (size_t)D.n_slots * D.Hkv * D.ctx_pad * D.hd * esz, true)
    }
    ALLOC(D.layers, const DevLayer*, sizeof(DevLayer) * c.n_layers, false)
    ALLOC(D.embed, const void*, V * d * esz, false)
    ALLOC(D.wlm, const uint4*, V * d * esz, false)
    ALLOC(D.g_final, const float*, d * 4, false)
    ALLOC(D.rope_cos, const float*, (size_t)D.ctx_pad * (D.hd / 2) * 4, false)
    ALLOC(D.rope_sin, const float*, (size_t)D.ctx_pad * (D.hd / 2) * 4, false)
    ALLOC(D.X, float*, kRows * d * 4, true)
    ALLOC(D.A, void*, kRows * d * 4, true)
    ALLOC(D.ssq, float*, (d / 16) * kRows * 4, true)
    ALLOC(D.Q_hi, void*, kRows * q * 4, true)
    ALLOC(D.Q_lo, void*, kRows * q * 4, true)
    const size_t pass_seqs = D.n_slots < kMaxSegs ? D.n_slots : kMaxSegs;
    const size_t att_part_bytes = pass_seqs * D.Hkv * D.max_chunks * D.G * kRows * (D.hd + 4) * 4;
    ALLOC(D.att_part, float*, att_part_bytes, true)
    const size_t xch_bytes = (size_t)D.d / 16 * kSplitWaysMax * 256 * 4;    // a partial tile per tile and K range
    ALLOC(D.xch, float*, xch_bytes, true)
    ALLOC(D.xch_ticket, int*, kSplitTickets * 4, true)
    ALLOC(D.O, void*, kRows * q * 4, true)
    ALLOC(D.H, void*, kRows * F * 4, true)
    ALLOC(D.logits, float*, kRows * V * 4, true)
    ALLOC(D.best_val, float*, (size_t)m->nwg * kRows * 4, true)
    ALLOC(D.best_idx, int*, (size_t)m->nwg * kRows * 4, true)
#undef ALLOC
    if (hipMemcpyAsync(const_cast<DevLayer*>(D.layers), m->layers_host.data(), sizeof(DevLayer) * c.n_layers,
                       hipMemcpyHostToDevice, m->stream) != hipSuccess)
        return bail(fail(AMUSD_E_HIP, "layer table upload"));
    if (hipHostMalloc(reinterpret_cast<void**>(&m->hstage), sizeof(HostStage), hipHostMallocDefault) != hipSuccess)
        return bail(fail(AMUSD_E_HIP, "pinned staging allocation"));
    std::memset(m->hstage, 0, sizeof(HostStage));
    // the acceptance kernel writes its 192-byte result straight into this pinned host block: no copy per pass
    {
        void* dev = nullptr;
        if (hipHostGetDevicePointer(&dev, m->hstage, 0) != hipSuccess)
            return bail(fail(AMUSD_E_HIP, "device address of the pinned result block"));
        D.res = reinterpret_cast<PassResult*>(dev);
    }
    if (hipEventCreate(&m->ev0) != hipSuccess || hipEventCreate(&m->ev1) != hipSuccess)
        return bail(fail(AMUSD_E_HIP, "event creation"));

    // rotary tables: angles in double, rounded once to fp32
    {
        const int half = D.hd / 2;
        std::vector<float> cs((size_t)D.ctx_pad * half), sn((size_t)D.ctx_pad * half);
        std::vector<double> inv(half);
        for (int i = 0; i < half; ++i) inv[i] = std::pow((double)c.rope_theta, -2.0 * i / D.hd);
        for (int pos = 0; pos < D.ctx_pad; ++pos)
            for (int i = 0; i < half; ++i) {
                const double a = (double)pos * inv[i];
                cs[(size_t)pos * half + i] = (float)std::cos(a);
                sn[(size_t)pos * half + i] = (float)std::sin(a);
            }
        if (hipMemcpy(const_cast<float*>(D.rope_cos), cs.data(), cs.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(const_cast<float*>(D.rope_sin), sn.data(), sn.size() * 4, hipMemcpyHostToDevice) != hipSuccess)
            return bail(fail(AMUSD_E_HIP, "rotary table upload"));
    }
    // The same workspace once more, inside the static scratch array (amusd_verify_static).
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        m->id = g_next_model_id++;
    }
    {
        void* base = nullptr;
        if (static_scratch_address(m->device, &base) != hipSuccess)
            return bail(fail(AMUSD_E_HIP, "address of the static scratch array"));
        m->dm_static = D;
        size_t off = 0;
        auto place = [&](size_t bytes) {
            void* p = static_cast<char*>(base) + off;
            off += (bytes + 255) & ~(size_t)255;
            return p;
        };
        DevModel& S = m->dm_static;
        S.X = static_cast<float*>(place(kRows * d * 4));
        S.A = place(kRows * d * 4);
        S.ssq = static_cast<float*>(place((d / 16) * kRows * 4));
        S.Q_hi = place(kRows * q * 4);
        S.Q_lo = place(kRows * q * 4);
        S.att_part = static_cast<float*>(place(att_part_bytes));
        S.xch = static_cast<float*>(place(xch_bytes));
        S.xch_ticket = static_cast<int*>(place(kSplitTickets * 4));
        S.O = place(kRows * q * 4);
        S.H = place(kRows * F * 4);
        S.best_val = static_cast<float*>(place((size_t)m->nwg * kRows * 4));
        S.best_idx = static_cast<int*>(place((size_t)m->nwg * kRows * 4));
        m->static_bytes = off;      // may exceed the array: amusd_verify_static then refuses the model
    }
    if (hipStreamSynchronize(m->stream) != hipSuccess) return bail(fail(AMUSD_E_HIP, "create: stream sync"));
    *out = m;
    return AMUSD_OK;
}

int amusd_model_set_tensor(amusd_model* m, int32_t id, int32_t layer, const void* data, int32_t on_device) {
    if (!m || !data) return fail(AMUSD_E_ARG, "null argument");
    if (id < 0 || id >= AMUSD_T_COUNT) return fail(AMUSD_E_ARG, "unknown tensor id");
    const amusd_config& c = m->cfg;
    const TensorInfo ti = tensor_info(c, id);
    if (ti.per_layer && (layer < 0 || layer >= c.n_layers)) return fail(AMUSD_E_ARG, "layer out of range");
    if (m->finalized) return fail(AMUSD_E_STATE, "model already finalized");
    const int esz = m->esz();
    const size_t bytes = (size_t)ti.rows * ti.cols * esz;
    const int slot = ti.per_layer ? layer + 1 : 0;
    DevModel& D = m->dm;

    if (ti.rows == 1) {   // gains -> fp32
        std::vector<char> raw(bytes);
        HIP_TRY(hipMemcpy(raw.data(), data, bytes, on_device ? hipMemcpyDeviceToHost : hipMemcpyHostToHost));
        std::vector<float> g(ti.cols);
        for (long i = 0; i < ti.cols; ++i)
            g[i] = esz == 2 ? bf16_bits_to_float(reinterpret_cast<const uint16_t*>(raw.data())[i])
                            : reinterpret_cast<const float*>(raw.data())[i];
        const float* dst = id == AMUSD_T_FINAL_NORM ? D.g_final
                           : id == AMUSD_T_NORM_ATTN ? m->layers_host[layer].g_attn
                                                     : m->layers_host[layer].g_mlp;
        HIP_TRY(hipMemcpy(const_cast<float*>(dst), g.data(), g.size() * 4, hipMemcpyHostToDevice));
        m->have[(size_t)id * (c.n_layers + 1) + slot] = 1;
        return AMUSD_OK;
    }
    if (id == AMUSD_T_EMBED) {
        HIP_TRY(hipMemcpy(const_cast<void*>(D.embed), data, bytes, on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice));
        m->have[(size_t)id * (c.n_layers + 1) + slot] = 1;
        return AMUSD_OK;
    }
    const void* src = data;
    if (!on_device) {
        if (m->staging_bytes < bytes) {
            if (m->staging) HIP_TRY(hipFree(m->staging));
            m->staging = nullptr;
            m->staging_bytes = 0;
            HIP_TRY(hipMalloc(&m->staging, bytes));
            m->staging_bytes = bytes;
        }
        HIP_TRY(hipMemcpy(m->staging, data, bytes, hipMemcpyHostToDevice));
        src = m->staging;
    }
    const int hd = c.head_dim;
    uint4* dst = nullptr;
    int n_tiles = (int)(ti.rows / 16), off = 0, kind = kNatural;
    switch (id) {
        case AMUSD_T_LM_HEAD: dst = const_cast<uint4*>(D.wlm); break;
        case AMUSD_T_WQ: dst = const_cast<uint4*>(m->layers_host[layer].wqkv); kind = kRopePairs; break;
        case AMUSD_T_WK: dst = const_cast<uint4*>(m->layers_host[layer].wqkv); kind = kRopePairs; off = D.qdim / 16; break;
        case AMUSD_T_WV: dst = const_cast<uint4*>(m->layers_host[layer].wqkv); off = (D.qdim + D.kvdim) / 16; break;
        case AMUSD_T_WO: dst = const_cast<uint4*>(m->layers_host[layer].wo); break;
        case AMUSD_T_WG: dst = const_cast<uint4*>(m->layers_host[layer].wgu); kind = kGate; n_tiles = (int)(ti.rows / 8); break;
        case AMUSD_T_WU: dst = const_cast<uint4*>(m->layers_host[layer].wgu); kind = kUp; n_tiles = (int)(ti.rows / 8); break;
        case AMUSD_T_WD: dst = const_cast<uint4*>(m->layers_host[layer].wd); break;
        default: return fail(AMUSD_E_ARG, "unknown tensor id");
    }
    HIP_TRY(launch_relayout(c.dtype, dst, src, (int)ti.cols, n_tiles, off, kind, hd, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    m->have[(size_t)id * (c.n_layers + 1) + slot] = 1;
    return AMUSD_OK;
}

int amusd_model_finalize(amusd_model* m) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    const amusd_config& c = m->cfg;
    for (int id = 0; id < AMUSD_T_COUNT; ++id) {
        const TensorInfo ti = tensor_info(c, id);
        const int lo = ti.per_layer ? 1 : 0, hi = ti.per_layer ? c.n_layers : 0;
        for (int s = lo; s <= hi; ++s)
            if (!m->have[(size_t)id * (c.n_layers + 1) + s])
                return fail(AMUSD_E_STATE, std::string("tensor not set: ") + kTensorNames[id] +
                                               (ti.per_layer ? " layer " + std::to_string(s - 1) : std::string()));
    }
    if (m->staging) {
        HIP_TRY(hipFree(m->staging));
        m->staging = nullptr;
        m->staging_bytes = 0;
    }
    m->finalized = true;
    return AMUSD_OK;
}

int amusd_model_load(const amusd_config* cfg, const amusd_weights* w, void* hip_stream, amusd_model** out) {
    if (!cfg || !w || !out) return fail(AMUSD_E_ARG, "null argument");
    if (!w->embed || !w->lm_head || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->wg || !w->wu ||
        !w->wd || !w->norm_attn || !w->norm_mlp)
        return fail(AMUSD_E_ARG, "null weight pointer");
    amusd_model* m = nullptr;
    int rc = amusd_model_create(cfg, hip_stream, &m);
    if (rc) return rc;
    auto set = [&](int id, int layer, const void* p) {
        if (rc == AMUSD_OK) rc = p ? amusd_model_set_tensor(m, id, layer, p, w->on_device) : fail(AMUSD_E_ARG, "null weight pointer");
    };
    set(AMUSD_T_EMBED, 0, w->embed);
    set(AMUSD_T_LM_HEAD, 0, w->lm_head);
    set(AMUSD_T_FINAL_NORM, 0, w->final_norm);
    for (int l = 0; l < cfg->n_layers; ++l) {
        set(AMUSD_T_WQ, l, w->wq[l]); set(AMUSD_T_WK, l, w->wk[l]); set(AMUSD_T_WV, l, w->wv[l]);
        set(AMUSD_T_WO, l, w->wo[l]); set(AMUSD_T_WG, l, w->wg[l]); set(AMUSD_T_WU, l, w->wu[l]);
        set(AMUSD_T_WD, l, w->wd[l]); set(AMUSD_T_NORM_ATTN, l, w->norm_attn[l]); set(AMUSD_T_NORM_MLP, l, w->norm_mlp[l]);
    }
    if (rc == AMUSD_OK) rc = amusd_model_finalize(m);
    if (rc) {
        const std::string keep = g_last_error;
        amusd_model_free(m);
        g_last_error = keep;
        return rc;
    }
    *out = m;
    return AMUSD_OK;
}

int amusd_model_free(amusd_model* m) {
    if (!m) return AMUSD_OK;
    if (m->stream || !m->allocs.empty()) (void)hipStreamSynchronize(m->stream);
    for (void* p : m->allocs) (void)hipFree(p);
    if (m->staging) (void)hipFree(m->staging);
    if (m->hstage) (void)hipHostFree(m->hstage);
    if (m->ev0) (void)hipEventDestroy(m->ev0);
    if (m->ev1) (void)hipEventDestroy(m->ev1);
    for (hipEvent_t e : m->tev_begin) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : m->tev_end) if (e) (void)hipEventDestroy(e);
    delete m;
    return AMUSD_OK;
}

int amusd_seq_prefill(amusd_model* m, int32_t seq, const int32_t* tokens, int32_t n, int32_t* next_token) {
    int rc = need_ready(m);
    if (rc || (rc = need_seq(m, seq))) return rc;
    if (!tokens || n < 1) return fail(AMUSD_E_ARG, "prefill: null tokens or n < 1");
    SeqState& q = m->seqs[seq];
    if ((long)q.kv_len + n > m->cfg.max_ctx) return fail(AMUSD_E_CAPACITY, "prefill: exceeds max_ctx");
    if ((rc = check_tokens(m, tokens, n))) return rc;
    // 16-bit models run fastest with at most 8 rows per pass (hi and lo halves share one operand fragment)
    const int chunk = m->cfg.dtype == AMUSD_DTYPE_BF16 && m->cfg.max_k > 8 ? 8 : m->cfg.max_k;
    const int len_before = q.kv_len, next_before = q.p_next;
    for (int s = 0; s < n; s += chunk) {
        const int k = n - s < chunk ? n - s : chunk;
        if ((rc = run_pass(m, seq, q.kv_len, tokens + s, k, true))) {
            q.kv_len = len_before;          // the passes that succeeded are dropped again: an O(1) truncation
            q.p_next = next_before;
            return rc;
        }
    }
    if (next_token) *next_token = q.p_next;
    return AMUSD_OK;
}

int amusd_prefill(amusd_model* m, const int32_t* tokens, int32_t n, int32_t* next_token) {
    return amusd_seq_prefill(m, 0, tokens, n, next_token);
}

static int verify_batch_impl(amusd_model* m, int32_t n_seq, const int32_t* seq_ids, const int32_t* ctx_len,
                             const int32_t* k, const int32_t* drafts, int32_t* accept_len, int32_t* next_token,
                             bool use_static) {
    int rc = need_ready(m);
    if (rc) return rc;
    if (use_static && m->static_bytes > kStaticScratchBytes)
        return fail(AMUSD_E_CAPACITY, "verify_static: this model's pass workspace (" + std::to_string(m->static_bytes) +
                                          " bytes) exceeds the static scratch array (" +
                                          std::to_string(kStaticScratchBytes) + " bytes)");
    if (!seq_ids || !ctx_len || !k || !drafts || !accept_len || !next_token)
        return fail(AMUSD_E_ARG, "verify_batch: null argument");
    if (n_seq < 1 || n_seq > kMaxSegs) return fail(AMUSD_E_ARG, "verify_batch: n_seq outside [1, 16]");
    SegReq segs[kMaxSegs];
    int rows = 0;
    for (int i = 0; i < n_seq; ++i) {
        if ((rc = need_seq(m, seq_ids[i]))) return rc;
        for (int j = 0; j < i; ++j)
            if (seq_ids[j] == seq_ids[i]) return fail(AMUSD_E_ARG, "verify_batch: a sequence appears twice");
        if (k[i] < 1) return fail(AMUSD_E_ARG, "verify_batch: k < 1");
        const SeqState& q = m->seqs[seq_ids[i]];
        if (ctx_len[i] < 0 || ctx_len[i] > q.kv_len) return fail(AMUSD_E_RANGE, "verify: ctx_len outside [0, kv_len]");
        if ((long)ctx_len[i] + k[i] > m->cfg.max_ctx) return fail(AMUSD_E_CAPACITY, "verify: ctx_len + k exceeds max_ctx");
        segs[i] = SegReq{seq_ids[i], ctx_len[i], drafts + rows, k[i]};
        rows += k[i];
        if (rows > m->cfg.max_k) return fail(AMUSD_E_ARG, "verify: more than max_k rows in one pass");
    }
    if ((rc = check_tokens(m, drafts, rows))) return rc;
    for (int i = 0; i < n_seq; ++i)
        if (m->seqs[seq_ids[i]].greedy_at[ctx_len[i]] < 0)
            return fail(AMUSD_E_STATE, "verify: the model's token for position ctx_len is unknown");
    if ((rc = run_pass(m, segs, n_seq, false, use_static))) return rc;
    for (int i = 0; i < n_seq; ++i) {
        accept_len[i] = m->hstage->res.accept_len[i];
        next_token[i] = m->hstage->res.next_token[i];
    }
    return AMUSD_OK;
}

int amusd_verify_batch(amusd_model* m, int32_t n_seq, const int32_t* seq_ids, const int32_t* ctx_len, const int32_t* k,
                       const int32_t* drafts, int32_t* accept_len, int32_t* next_token) {
    return verify_batch_impl(m, n_seq, seq_ids, ctx_len, k, drafts, accept_len, next_token, false);
}

int amusd_verify_static(amusd_model* m, int32_t ctx_len, const int32_t* draft, int32_t k, int32_t* accept_len,
                        int32_t* next_token) {
    int rc = need_ready(m);
    if (rc) return rc;
    if (!draft || !accept_len || !next_token) return fail(AMUSD_E_ARG, "verify_static: null argument");
    if (k < 1 || k > m->cfg.max_k) return fail(AMUSD_E_ARG, "verify_static: k outside [1, max_k]");
    const int32_t seq = 0;
    return verify_batch_impl(m, 1, &seq, &ctx_len, &k, draft, accept_len, next_token, true);
}

int64_t amusd_static_scratch_bytes(const amusd_model* m) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    return (int64_t)m->static_bytes;
}

int amusd_verify(amusd_model* m, int32_t ctx_len, const int32_t* draft, int32_t k, int32_t* accept_len,
                 int32_t* next_token) {
    int rc = need_ready(m);
    if (rc) return rc;
    if (!draft || !accept_len || !next_token) return fail(AMUSD_E_ARG, "verify: null argument");
    if (k < 1 || k > m->cfg.max_k) return fail(AMUSD_E_ARG, "verify: k outside [1, max_k]");
    const int32_t seq = 0;
    return amusd_verify_batch(m, 1, &seq, &ctx_len, &k, draft, accept_len, next_token);
}

int amusd_draft_step_batch(amusd_model* m, int32_t n_seq, const int32_t* seq_ids, int32_t* tokens_out) {
    int rc = need_ready(m);
    if (rc) return rc;
    if (!seq_ids || !tokens_out) return fail(AMUSD_E_ARG, "draft_step: null argument");
    if (n_seq < 1 || n_seq > kMaxSegs || n_seq > m->cfg.max_k) return fail(AMUSD_E_ARG, "draft_step: n_seq outside [1, max_k]");
    SegReq segs[kMaxSegs];
    int32_t toks[kMaxSegs];
    for (int i = 0; i < n_seq; ++i) {
        if ((rc = need_seq(m, seq_ids[i]))) return rc;
        for (int j = 0; j < i; ++j)
            if (seq_ids[j] == seq_ids[i]) return fail(AMUSD_E_ARG, "draft_step: a sequence appears twice");
        const SeqState& q = m->seqs[seq_ids[i]];
        if (q.p_next < 0) return fail(AMUSD_E_STATE, "draft_step: p_next unknown");
        if (q.kv_len + 1 > m->cfg.max_ctx) return fail(AMUSD_E_CAPACITY, "draft_step: cache full");
        toks[i] = q.p_next;
        segs[i] = SegReq{seq_ids[i], q.kv_len, &toks[i], 1};
    }
    if ((rc = run_pass(m, segs, n_seq, true))) return rc;
    for (int i = 0; i < n_seq; ++i) tokens_out[i] = m->seqs[seq_ids[i]].p_next;
    return AMUSD_OK;
}

int amusd_draft_step(amusd_model* m, int32_t* token_out) {
    const int32_t seq = 0;
    return amusd_draft_step_batch(m, 1, &seq, token_out);
}

int amusd_seq_rollback(amusd_model* m, int32_t seq, int32_t new_len) {
    int rc = need_seq(m, seq);
    if (rc) return rc;
    SeqState& q = m->seqs[seq];
    if (new_len < 0 || new_len > q.kv_len) return fail(AMUSD_E_RANGE, "rollback: new_len outside [0, kv_len]");
    q.kv_len = new_len;
    q.p_next = q.greedy_at[new_len];
    return AMUSD_OK;
}

int amusd_kv_rollback(amusd_model* m, int32_t new_len) { return amusd_seq_rollback(m, 0, new_len); }

int amusd_seq_set_next(amusd_model* m, int32_t seq, int32_t token) {
    int rc = need_seq(m, seq);
    if (rc) return rc;
    if (token < 0 || token >= m->cfg.vocab) return fail(AMUSD_E_TOKEN, "set_next: token id outside [0, vocab)");
    SeqState& q = m->seqs[seq];
    q.p_next = token;
    q.greedy_at[q.kv_len] = token;
    return AMUSD_OK;
}

int amusd_set_next(amusd_model* m, int32_t token) { return amusd_seq_set_next(m, 0, token); }

int amusd_seq_len(const amusd_model* m, int32_t seq) {
    const int rc = need_seq(m, seq);
    return rc ? rc : m->seqs[seq].kv_len;
}

int amusd_kv_len(const amusd_model* m) { return amusd_seq_len(m, 0); }

int amusd_seq_get_next(const amusd_model* m, int32_t seq, int32_t* token) {
    if (!token) return fail(AMUSD_E_ARG, "null argument");
    const int rc = need_seq(m, seq);
    if (rc) return rc;
    *token = m->seqs[seq].p_next;
    return AMUSD_OK;
}

int amusd_get_next(const amusd_model* m, int32_t* token) { return amusd_seq_get_next(m, 0, token); }

int amusd_set_option(amusd_model* m, int32_t option, int32_t value) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    switch (option) {
        case AMUSD_OPT_KEEP_LOGITS: m->keep_logits = value != 0; return AMUSD_OK;
        case AMUSD_OPT_TIME_STAGE: {
            if (value < -1 || value >= AMUSD_STAGE_COUNT) return fail(AMUSD_E_ARG, "unknown stage");
            if (value >= 0 && m->tev_begin.empty()) {
                m->tev_begin.resize(m->cfg.n_layers);
                m->tev_end.resize(m->cfg.n_layers);
                for (int i = 0; i < m->cfg.n_layers; ++i) {
                    HIP_TRY(hipEventCreate(&m->tev_begin[i]));
                    HIP_TRY(hipEventCreate(&m->tev_end[i]));
                }
                m->timer.begin = m->tev_begin.data();
                m->timer.end = m->tev_end.data();
            }
            m->timer.stage = value;
            m->stage_ms = 0.0;
            m->stage_launches = 0;
            return AMUSD_OK;
        }
        default: return fail(AMUSD_E_ARG, "unknown option");
    }
}

int amusd_get_logits(amusd_model* m, float* out, int32_t rows) {
    int rc = need_ready(m);
    if (rc) return rc;
    if (!out || rows < 1 || rows > kRows) return fail(AMUSD_E_ARG, "get_logits: bad argument");
    if (!m->logits_valid || rows > m->last_rows) return fail(AMUSD_E_STATE, "get_logits: the last pass kept no such logits");
    HIP_TRY(hipMemcpy(out, m->dm.logits, (size_t)rows * m->cfg.vocab * 4, hipMemcpyDeviceToHost));
    return AMUSD_OK;
}

int amusd_get_greedy(amusd_model* m, int32_t* out, int32_t rows) {
    int rc = need_ready(m);
    if (rc) return rc;
    if (!out || rows < 1 || rows > m->last_rows) return fail(AMUSD_E_ARG, "get_greedy: bad argument");
    for (int j = 0; j < rows; ++j) out[j] = m->hstage->res.greedy[j];
    return AMUSD_OK;
}

int amusd_last_pass_ms(amusd_model* m, float* ms) {
    if (!m || !ms) return fail(AMUSD_E_ARG, "null argument");
    *ms = m->last_ms;
    return AMUSD_OK;
}

int amusd_stage_time(amusd_model* m, double* total_ms, int64_t* launches, int64_t* bytes_per_launch) {
    if (!m || !total_ms || !launches || !bytes_per_launch) return fail(AMUSD_E_ARG, "null argument");
    if (m->timer.stage < 0) return fail(AMUSD_E_STATE, "no stage selected for timing");
    const amusd_config& c = m->cfg;
    const int64_t d = c.d_model, q = (int64_t)c.n_q_heads * c.head_dim, kv = (int64_t)c.n_kv_heads * c.head_dim,
                  F = c.d_ffn, V = c.vocab, e = m->esz();
    int64_t b = 0;
    switch (m->timer.stage) {
        case AMUSD_STAGE_QKV: b = d * (q + 2 * kv) * e; break;
        case AMUSD_STAGE_ATTENTION: b = 2 * kv * e * m->last_positions; break;
        case AMUSD_STAGE_OPROJ: b = q * d * e; break;
        case AMUSD_STAGE_GATEUP: b = 2 * d * F * e; break;
        case AMUSD_STAGE_DOWN: b = d * F * e; break;
        case AMUSD_STAGE_LMHEAD: b = V * d * e; break;
        default: b = 0;
    }
    *total_ms = m->stage_ms;
    *launches = m->stage_launches;
    *bytes_per_launch = b;
    return AMUSD_OK;
}

int amusd_get_kv(amusd_model* m, int32_t layer, int32_t which, int32_t pos0, int32_t n, float* out) {
    return amusd_seq_get_kv(m, 0, layer, which, pos0, n, out);
}

int amusd_seq_get_kv(amusd_model* m, int32_t seq, int32_t layer, int32_t which, int32_t pos0, int32_t n, float* out) {
    int rc = need_ready(m);
    if (rc || (rc = need_seq(m, seq))) return rc;
    const DevModel& D = m->dm;
    if (!out || layer < 0 || layer >= D.n_layers || (which != 0 && which != 1) || pos0 < 0 || n < 1 || pos0 + n > D.ctx_pad)
        return fail(AMUSD_E_ARG, "get_kv: bad argument");
    const int esz = m->esz(), hd = D.hd, BK = m->block_keys(), EPL = 16 / esz;
    const size_t elems = (size_t)D.Hkv * D.ctx_pad * hd;
    std::vector<char> raw(elems * esz);
    const char* cache = reinterpret_cast<const char*>(which ? m->layers_host[layer].vcache : m->layers_host[layer].kcache);
    HIP_TRY(hipMemcpy(raw.data(), cache + (size_t)seq * raw.size(), raw.size(), hipMemcpyDeviceToHost));
    auto val = [&](size_t i) {   // the cache of a 16-bit model holds IEEE half
        return esz == 2 ? half_bits_to_float(reinterpret_cast<const uint16_t*>(raw.data())[i])
                        : reinterpret_cast<const float*>(raw.data())[i];
    };
    for (int h = 0; h < D.Hkv; ++h)
        for (int j = 0; j < n; ++j)
            for (int c = 0; c < hd; ++c) {
                const int pos = pos0 + j;
                size_t idx;
                if (!which) {
                    const int q4 = hd / 4, g = c / q4, w = c % q4;
                    idx = (size_t)h * D.ctx_pad * hd +
                          ((((size_t)(pos >> 4) * (q4 / EPL) + w / EPL) * 64) + g * 16 + (pos & 15)) * EPL + w % EPL;
                } else {
                    const int b = pos / BK, q = pos % BK;
                    const int e = (q / 16) * 4 + (q % 4), gg = (q % 16) / 4;
                    const size_t blk = ((size_t)h * (D.ctx_pad / BK) + b) * (hd / 16) + c / 16;
                    idx = (blk * 64 + gg * 16 + c % 16) * EPL + e;
                }
                out[((size_t)h * n + j) * hd + c] = val(idx);
            }
    return AMUSD_OK;
}

int64_t amusd_weight_bytes_per_pass(const amusd_model* m) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    const amusd_config& c = m->cfg;
    const int64_t d = c.d_model, q = (int64_t)c.n_q_heads * c.head_dim, kv = (int64_t)c.n_kv_heads * c.head_dim,
                  F = c.d_ffn, V = c.vocab;
    const int64_t per_layer = d * (q + 2 * kv) + q * d + 3 * d * F + 2 * d;
    return (c.n_layers * per_layer + V * d + d) * m->esz();
}

int64_t amusd_kv_bytes_per_pass(const amusd_model* m, int32_t ctx_len, int32_t k) {
    if (!m) return fail(AMUSD_E_ARG, "null model");
    const amusd_config& c = m->cfg;
    return (int64_t)c.n_layers * 2 * c.n_kv_heads * c.head_dim * m->esz() * ((int64_t)ctx_len + k);
}

int amusd_calibration_copy(void* dst, const void* src, int64_t bytes, void* hip_stream) {
    if (!dst || !src || bytes < 16 || bytes % 16) return fail(AMUSD_E_ARG, "calibration_copy: bad argument");
    HIP_TRY(launch_copy(reinterpret_cast<uint4*>(dst), reinterpret_cast<const uint4*>(src), (size_t)bytes / 16,
                        reinterpret_cast<hipStream_t>(hip_stream)));
    return AMUSD_OK;
}

int amusd_calibration_chain(const void* buf, int64_t buf_bytes, int64_t bytes_per_kernel, int32_t n_kernels, void* scratch,
                            void* hip_stream) {
    const int64_t unit = (int64_t)256 * kThreads * 16;       // one 16-byte load of every thread of every workgroup
    if (!buf || !scratch || n_kernels < 1 || bytes_per_kernel < unit || bytes_per_kernel % unit ||
        buf_bytes < bytes_per_kernel)
        return fail(AMUSD_E_ARG, "calibration_chain: bytes_per_kernel must be a positive multiple of 2 MiB and fit the buffer");
    float* io = reinterpret_cast<float*>(scratch);
    HIP_TRY(launch_stream_chain(reinterpret_cast<const uint4*>(buf), (size_t)buf_bytes / 16, (size_t)bytes_per_kernel / 16,
                                n_kernels, io, reinterpret_cast<unsigned*>(io + 512), reinterpret_cast<hipStream_t>(hip_stream)));
    return AMUSD_OK;
}

// ---- drivers ------------------------------------------------------------------------------------

namespace {
struct ModelBackend final : StepBackend {
    amusd_model* m;
    explicit ModelBackend(amusd_model* mm) : m(mm) {}
    int prefill(const int32_t* t, int n, int32_t* next) override { return amusd_prefill(m, t, n, next); }
    int verify(int ctx, const int32_t* d, int k, int32_t* acc, int32_t* next) override {
        return amusd_verify(m, ctx, d, k, acc, next);
    }
    int draft_step(int32_t* t) override { return amusd_draft_step(m, t); }
    int rollback(int n) override { return amusd_kv_rollback(m, n); }
    int set_next(int32_t t) override { return amusd_set_next(m, t); }
    int kv_len() const override { return m->seqs[0].kv_len; }
    int max_ctx() const override { return m->cfg.max_ctx; }
    int vocab() const override { return m->cfg.vocab; }
};

void export_stats(const LoopStats& s, amusd_loop_stats* out) {
    if (!out) return;
    out->rounds = s.rounds;
    out->rollbacks = s.rollbacks;
    out->draft_steps = s.draft_steps;
    out->accepted_total = s.accepted_total;
    for (int i = 0; i <= AMUSD_MAX_K; ++i) out->accept_hist[i] = s.accept_hist[i];
    out->wall_ms = s.wall_ms;
}

int check_loop_args(const int32_t* prompt, int n_prompt, int n_new, int k_max, const int32_t* out) {
    if (!prompt || !out || n_prompt < 1 || n_new < 1) return fail(AMUSD_E_ARG, "generate: bad argument");
    if (k_max < 1 || k_max > AMUSD_MAX_K) return fail(AMUSD_E_ARG, "generate: k_max outside [1,16]");
    return AMUSD_OK;
}
}  // namespace

int amusd_generate_async(amusd_model* draft, amusd_model* verify, const int32_t* prompt, int32_t n_prompt, int32_t n_new,
                         int32_t k_max, int32_t* out_tokens, amusd_loop_stats* stats) {
    int rc = need_ready(draft);
    if (rc || (rc = need_ready(verify))) return rc;
    if ((rc = check_loop_args(prompt, n_prompt, n_new, k_max, out_tokens))) return rc;
    if (draft == verify) return fail(AMUSD_E_ARG, "generate_async: draft and verify must be different models");
    if (draft->cfg.vocab != verify->cfg.vocab) return fail(AMUSD_E_ARG, "generate_async: vocabularies differ");
    if (k_max > verify->cfg.max_k) return fail(AMUSD_E_ARG, "generate_async: k_max exceeds the verify model's max_k");
    ModelBackend d(draft), v(verify);
    LoopStats s;
    rc = run_async(d, v, prompt, n_prompt, n_new, k_max, out_tokens, &s);
    export_stats(s, stats);
    return rc;
}

int amusd_generate_sync(amusd_model* draft, amusd_model* verify, const int32_t* prompt, int32_t n_prompt, int32_t n_new,
                        int32_t k_max, int32_t* out_tokens, amusd_loop_stats* stats) {
    int rc = need_ready(draft);
    if (rc || (rc = need_ready(verify))) return rc;
    if ((rc = check_loop_args(prompt, n_prompt, n_new, k_max, out_tokens))) return rc;
    if (draft == verify) return fail(AMUSD_E_ARG, "generate_sync: draft and verify must be different models");
    if (draft->cfg.vocab != verify->cfg.vocab) return fail(AMUSD_E_ARG, "generate_sync: vocabularies differ");
    if (k_max > verify->cfg.max_k) return fail(AMUSD_E_ARG, "generate_sync: k_max exceeds the verify model's max_k");
    ModelBackend d(draft), v(verify);
    LoopStats s;
    rc = run_sync(d, v, prompt, n_prompt, n_new, k_max, out_tokens, &s);
    export_stats(s, stats);
    return rc;
}

int amusd_generate_greedy(amusd_model* m, const int32_t* prompt, int32_t n_prompt, int32_t n_new, int32_t* out_tokens,
                          amusd_loop_stats* stats) {
    int rc = need_ready(m);
    if (rc) return rc;
    if ((rc = check_loop_args(prompt, n_prompt, n_new, 1, out_tokens))) return rc;
    ModelBackend b(m);
    LoopStats s;
    rc = run_greedy(b, prompt, n_prompt, n_new, out_tokens, &s);
    export_stats(s, stats);
    return rc;
}

}  // extern "C"
