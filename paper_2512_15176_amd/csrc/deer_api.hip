// Host side of libdeer: context, buffer carving, call-order state machine, kernel launches.
// The C ABI is declared in include/deer.h.  Nothing here allocates device memory.
#include "deer_kernels.hpp"
#include "deer_tiled.hpp"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "deer.h"

using namespace deer;

// Scratch of deer_accept_and_commit_static, the entry point that allocates nothing: the per-share candidates of the
// sampling acceptance kernel (ACC_NB entries per sequence) followed by one arrival counter per sequence.  Every GPU
// the library runs on holds its own copy until the process ends.
constexpr int STATIC_MAX_BATCH = 64;
constexpr size_t STATIC_PART_BYTES = (size_t)STATIC_MAX_BATCH * ACC_NB * sizeof(AccPart);
constexpr size_t STATIC_SCRATCH_BYTES = STATIC_PART_BYTES + (size_t)STATIC_MAX_BATCH * sizeof(int);
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
// The array's name is a host-side stand-in, not a device address: host code uses the address that
// hipGetSymbolAddress gives, resolved once per device (with that device current) by deer_init_models.
constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES] = {};

namespace {

thread_local std::string g_init_error;


constexpr int STAMP_MAX_BLOCKS = 4096;   // workgroups whose stamps deer_debug_gemm_stamps can record (8 stamps each)
// rows of a prefill chunk / 32: dense models take 4096 rows per pass through the LDS-tiled GEMM, mixtures 512
// (their grouped expert buffers grow with the rows of a pass)
constexpr int PREFILL_TILES_DENSE = 128, PREFILL_TILES_MOE = 16;
int prefill_tiles(const deer_init_params &p) { return (p.target.n_experts || p.drafter.n_experts) ? PREFILL_TILES_MOE : PREFILL_TILES_DENSE; }
constexpr int PART_TILES_MIN = 16;   // split-K partials exist for passes of up to max(2 * batch, 16) row tiles
constexpr int MAX_NS = 32;          // key-range splits of block attention
constexpr int NARROW_MAX_D = 1024;  // residual width up to which a dense model's O projection runs in 32-column workgroups
constexpr int NEXT_SPAN_BYTES = 16 << 10;      // fetched ahead per 32-column block of a next-launch workgroup (4 blocks: 8 loads per thread)
constexpr int KV_FETCH_MAX_BYTES = 1 << 20;    // fetched ahead per kv head of K and of V^T: a share of one XCD's 4 MB L2
constexpr int ATT_HEAD_MAX_TILES = 12;   // per-head attention: most key tiles one wave may have to go through (equal or better up to 9, measured)
constexpr size_t PART_COLS = 131072; // fp32 columns of split-K partials per row (S * N <= PART_COLS)

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct ModelRT {
    deer_model_cfg c{};
    int n_qkv = 0, kattn = 0, F = 0;   // fused QKV width, Hq*hd, FFN width used by GEMMs
    int ssq_sub = 1;   // sums of squares of the residual stream per 128-column group (1) or per 32-column block (4)
    // weights (device)
    char *w = nullptr;
    size_t off_embed = 0, off_lm = 0, off_layers = 0, layer_bytes = 0;
    size_t lo_qkv = 0, lo_o = 0, lo_gu = 0, lo_d = 0;   // offsets inside a layer (gu/d: expert 0 for a mixture)
    size_t lo_router = 0, exp_gu_bytes = 0, exp_d_bytes = 0;   // mixture: router, per-expert matrix sizes
    size_t weight_bytes = 0;
    // kv (device, elements of bf16)
    uint16_t *kv = nullptr;
    size_t kv_k_base = 0, kv_v_base = 0, kv_layer_stride = 0, kv_seq_stride = 0, kv_head_stride = 0;
    size_t kv_bytes = 0;
    double *theta = nullptr;           // device [hd/2]
};

struct Work {   // carved from the workspace
    SeqState st{};
    RowMeta rm{};
    float2 *cs = nullptr;
    float *h = nullptr, *ssq = nullptr, *part = nullptr;
    uint4 *xa_hi = nullptr, *xa_lo = nullptr, *xb_hi = nullptr, *xb_lo = nullptr, *q_hi = nullptr, *q_lo = nullptr;
    float *opart = nullptr;
    float *logits[2] = {nullptr, nullptr};
    RowStat *stat = nullptr;
    RowResult *res[2] = {nullptr, nullptr};
    AcceptOut ao{};
    int *ids = nullptr;                // prompt staging [max_seq]
    // mixture-of-experts routing and staging (target only)
    int *route_e = nullptr, *exp_cnt = nullptr, *pair_row = nullptr, *pair_slot = nullptr;
    float *route_w = nullptr, *moe_out = nullptr;
    unsigned long long *moe_touched = nullptr;   // (layer, expert) pairs streamed since the last read
    uint4 *act_hi = nullptr, *act_lo = nullptr;
    int *gemm_cnt = nullptr, *attn_cnt = nullptr;   // arrival counters, zero between kernels
    size_t cnt_bytes = 0; char *cnt_base = nullptr;
    double *theta[2] = {nullptr, nullptr};
    size_t part_floats = 0;   // capacity of `part`
    AccPart *acc_part = nullptr; int *acc_cnt = nullptr;   // sampling acceptance: per-share candidates, arrival counters
    int4 *pf_desc = nullptr;  // prefill: per-tile (sequence, first position, rows, offset into ids)
    unsigned long long *stamps = nullptr;   // [STAMP_MAX_BLOCKS][8], written on request (deer_debug_gemm_stamps)
    size_t bytes = 0;
};

enum State { ST_INIT = 0, ST_PREFILLED, ST_DRAFTED, ST_VERIFIED };

}  // namespace

struct deer_ctx {
    deer_init_params p{};
    ModelRT m[2];
    Work wk;
    hipStream_t stream = nullptr;
    State state = ST_INIT;
    int batch = 0;
    int cur_k = 0;
    float cur_T = 0.f;
    int max_tiles = 0;
    int tiled_min_tiles = 128;       // the LDS-tiled GEMM runs where a launch has at least this many 256 x 256 tiles; 0: never
    // deer_debug_gemm_stamps: which streaming-GEMM launch of which model's passes records its stamps
    int stamp_model = 0, stamp_launch = -1, stamp_blocks = 0, gemm_launch_idx = 0, cur_pass_model = 0;
    int route_spread = 0;            // deer_debug_route_spread: synthetic uniform routing for mixture models
    int bonus = 0;                   // 1: verify k + 1 rows, commit one more target token after k accepted drafts
    void *static_scratch = nullptr;  // this device's copy of `scratch`
    const int *wk_draft = nullptr;   // draft buffer of the last verify_block
    std::vector<int> h_len, h_ing_n, h_finished;
    std::vector<char> h_ao;          // host staging of the acceptance results (pageable; used only if pinning failed)
    char *h_pin = nullptr;           // the same, page-locked: the copy lands without an intermediate staging copy
    size_t h_pin_bytes = 0;
    std::string err;
    // optional per-launch timing (deer_debug_profile)
    bool prof_on = false;
    struct ProfRec { int cls; hipEvent_t a, b; double bytes; int launches; };
    std::vector<ProfRec> prof;
    int prof_open_cls = -1;          // a run of consecutive launches of one class is being timed
    hipEvent_t prof_open_a = nullptr;
    double prof_open_bytes = 0.0;
    int prof_open_launches = 0;
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
};

namespace {

int fail(deer_ctx *c, int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf; else g_init_error = buf;
    return code;
}

hipEvent_t prof_event(deer_ctx *c) {
    if (c->ev_used == c->ev_pool.size()) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        c->ev_pool.push_back(e);
    }
    return c->ev_pool[c->ev_used++];
}

// Timing of launches when profiling is on.  Launches of one class that follow each other directly on the stream (the
// O, gate/up and down projections and the next layer's QKV projection) share one pair of events: an event between
// two of them costs more than the gap it would measure.  prof_close() ends the run that is open; it is called before
// a launch of another class, before every launch that is not timed, and before the records are read.
void prof_close(deer_ctx *c) {
    if (c->prof_open_cls < 0) return;
    hipEvent_t b = prof_event(c);
    if (b) {
        (void)hipEventRecord(b, c->stream);
        c->prof.push_back({c->prof_open_cls, c->prof_open_a, b, c->prof_open_bytes, c->prof_open_launches});
    }
    c->prof_open_cls = -1;
}
struct ProfScope {
    ProfScope(deer_ctx *c, int cls, double bytes) {
        if (!c->prof_on) return;
        if (c->prof_open_cls != cls) {
            prof_close(c);
            hipEvent_t a = prof_event(c);
            if (!a) return;
            (void)hipEventRecord(a, c->stream);
            c->prof_open_cls = cls; c->prof_open_a = a; c->prof_open_bytes = 0.0; c->prof_open_launches = 0;
        }
        c->prof_open_bytes += bytes;
        c->prof_open_launches += 1;
    }
};

#define HIPCHK(c, expr)                                                                            \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail((c), DEER_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define LAUNCHCHK(c, name)                                                                          \
    do {                                                                                            \
        hipError_t e_ = hipGetLastError();                                                          \
        if (e_ != hipSuccess) return fail((c), DEER_EHIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

const char *check_model(const deer_model_cfg &c) {
    if (c.n_layers < 1 || c.d_model < 128 || c.vocab < 128) return "n_layers/d_model/vocab too small";
    if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128) return "head_dim must be 32, 64 or 128";
    if (c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads) return "n_q_heads must be a multiple of n_kv_heads";
    if (c.d_model % CG) return "d_model must be a multiple of 128";
    if (c.d_model > 8192) return "d_model above 8192 is not supported (64 column groups of sums of squares per row)";
    if (((c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim) % CG) return "fused QKV width must be a multiple of 128";
    if ((c.n_q_heads * c.head_dim) % 16) return "n_q_heads*head_dim must be a multiple of 16";
    if (c.vocab % CG) return "vocab must be a multiple of 128";
    if (c.n_experts) {
        if (c.n_experts > 128 || c.top_k < 1 || c.top_k > 8 || c.top_k > c.n_experts) return "mixture needs n_experts <= 128 and 1 <= top_k <= 8";
        if (c.d_ff_expert < 64 || c.d_ff_expert % 64) return "d_ff_expert must be a multiple of 64";
    } else if (c.d_ff < 64 || c.d_ff % 64) return "d_ff must be a multiple of 64";
    if (!(c.rope_base > 1.f) || !(c.rms_eps >= 0.f)) return "bad rope_base / rms_eps";
    return nullptr;
}

void plan_model(ModelRT &m, const deer_model_cfg &c, int max_batch, int max_seq) {
    m.c = c;
    m.n_qkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    m.kattn = c.n_q_heads * c.head_dim;
    m.F = c.n_experts ? c.d_ff_expert : c.d_ff;
    // a small dense model runs its unsplit residual GEMMs in 32-column workgroups (k_gemm_resid32)
    m.ssq_sub = (!c.n_experts && c.d_model <= NARROW_MAX_D) ? 4 : 1;
    size_t d = c.d_model;
    m.off_embed = 0;
    m.off_lm = align_up((size_t)c.vocab * d * 2);
    m.off_layers = m.off_lm + align_up(d * (size_t)c.vocab * 2);
    m.lo_qkv = 0;
    m.lo_o = m.lo_qkv + align_up(d * m.n_qkv * 2);
    m.lo_router = m.lo_o + align_up((size_t)m.kattn * d * 2);
    m.lo_gu = m.lo_router + (c.n_experts ? align_up(d * CG * 2) : 0);
    m.exp_gu_bytes = align_up(d * 2 * m.F * 2);
    m.exp_d_bytes = align_up((size_t)m.F * d * 2);
    const size_t ne = c.n_experts ? c.n_experts : 1;
    m.lo_d = m.lo_gu + m.exp_gu_bytes * ne;
    m.layer_bytes = m.lo_d + m.exp_d_bytes * ne;
    m.weight_bytes = m.off_layers + m.layer_bytes * c.n_layers;
    m.kv_head_stride = (size_t)max_seq * c.head_dim;
    m.kv_seq_stride = m.kv_head_stride * c.n_kv_heads;
    m.kv_layer_stride = m.kv_seq_stride * max_batch;
    m.kv_k_base = 0;
    m.kv_v_base = m.kv_layer_stride * c.n_layers;
    m.kv_bytes = align_up(2 * m.kv_layer_stride * c.n_layers * 2);
}

// Carves the workspace; with base == nullptr only computes the size.
void plan_work(Work &w, const deer_init_params &p, char *base) {
    const int B = p.max_batch;
    const int MAXT = std::max(2 * B, prefill_tiles(p)), MAXR = MAXT * 32;
    const int PARTR = std::max(2 * B, PART_TILES_MIN) * 32;
    const deer_model_cfg &t = p.target, &d = p.drafter;
    const size_t dmax = std::max(t.d_model, d.d_model);
    const size_t kattn = std::max(t.n_q_heads * t.head_dim, d.n_q_heads * d.head_dim);
    const size_t fmax = std::max(t.n_experts ? t.d_ff_expert : t.d_ff, d.n_experts ? d.d_ff_expert : d.d_ff);
    const size_t kb = std::max(kattn, fmax);
    const size_t hq = std::max(t.n_q_heads, d.n_q_heads);
    const size_t hdmax = std::max(t.head_dim, d.head_dim);
    const size_t V = std::max(t.vocab, d.vocab);
    const size_t lmrows = (size_t)B * 32;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return base ? base + o : nullptr; };
    w.st.len = (int *)take(B * 4); w.st.dr_len = (int *)take(B * 4); w.st.pending = (int *)take(B * 4);
    w.st.ing_n = (int *)take(B * 4); w.st.finished = (int *)take(B * 4); w.st.ing_tok = (int *)take((size_t)B * 32 * 4);
    w.rm.tok = (int *)take(MAXR * 4); w.rm.pos = (int *)take(MAXR * 4); w.rm.limit = (int *)take(MAXR * 4);
    w.rm.slot = (int *)take(MAXR * 4); w.rm.tile_seq = (int *)take(MAXT * 4);
    w.cs = (float2 *)take((size_t)MAXR * 64 * sizeof(float2));
    w.theta[0] = (double *)take(64 * 8); w.theta[1] = (double *)take(64 * 8);
    w.h = (float *)take((size_t)MAXR * dmax * 4);
    w.ssq = (float *)take((size_t)MAXR * std::max<size_t>(dmax / CG, std::min<size_t>(dmax, NARROW_MAX_D) / 32) * 4);
    w.xa_hi = (uint4 *)take((size_t)MAXT * (dmax / 16) * 1024); w.xa_lo = (uint4 *)take((size_t)MAXT * (dmax / 16) * 1024);
    w.xb_hi = (uint4 *)take((size_t)MAXT * (kb / 16) * 1024); w.xb_lo = (uint4 *)take((size_t)MAXT * (kb / 16) * 1024);
    w.q_hi = (uint4 *)take((size_t)MAXT * (kattn / 16) * 1024); w.q_lo = (uint4 *)take((size_t)MAXT * (kattn / 16) * 1024);
    w.part = (float *)take((size_t)PARTR * PART_COLS * 4); w.part_floats = (size_t)PARTR * PART_COLS;
    w.opart = (float *)take((size_t)std::max(64, MAXT) * hq * (32 * hdmax + 64) * 4);
    w.logits[0] = (float *)take(lmrows * V * 4); w.logits[1] = (float *)take(lmrows * V * 4);
    w.stat = (RowStat *)take(lmrows * (V / CG) * sizeof(RowStat));
    w.res[0] = (RowResult *)take(lmrows * sizeof(RowResult)); w.res[1] = (RowResult *)take(lmrows * sizeof(RowResult));
    w.ao.accept_len = (int *)take(B * 4); w.ao.n_committed = (int *)take(B * 4); w.ao.committed = (int *)take((size_t)B * 32 * 4);
    w.acc_part = (AccPart *)take((size_t)B * ACC_NB * sizeof(AccPart));
    w.ids = (int *)take((size_t)B * p.max_seq * 4);
    w.pf_desc = (int4 *)take((size_t)MAXT * sizeof(int4));
    for (const deer_model_cfg *mc : {&t, &d}) {
        if (!mc->n_experts || w.route_e) continue;
        const size_t chunks = MAXT;   // 32-pair chunks per expert: at most every row of the pass
        w.route_e = (int *)take((size_t)MAXR * 8 * 4); w.route_w = (float *)take((size_t)MAXR * 8 * 4);
        w.exp_cnt = (int *)take(128 * 4); w.moe_touched = (unsigned long long *)take(8);
        w.pair_row = (int *)take((size_t)128 * MAXR * 4); w.pair_slot = (int *)take((size_t)128 * MAXR * 4);
        w.moe_out = (float *)take((size_t)MAXR * 8 * dmax * 4);
        w.act_hi = (uint4 *)take((size_t)128 * chunks * (fmax / 16) * 1024); w.act_lo = (uint4 *)take((size_t)128 * chunks * (fmax / 16) * 1024);
    }
    {
        const size_t ng = (size_t)(std::max(std::max(t.d_model, d.d_model), 4 * (int)fmax) / CG + 64) * MAXT, na = (size_t)MAXT * hq;
        w.cnt_base = take((ng + na + (size_t)B) * 4);
        w.gemm_cnt = (int *)w.cnt_base;
        w.attn_cnt = w.gemm_cnt ? w.gemm_cnt + ng : nullptr;
        w.acc_cnt = w.gemm_cnt ? w.gemm_cnt + ng + na : nullptr;
        w.cnt_bytes = (ng + na + (size_t)B) * 4;
    }
    w.stamps = (unsigned long long *)take((size_t)STAMP_MAX_BLOCKS * 8 * 8);
    w.bytes = off;
}

const char *check_params(const deer_init_params *p) {
    if (!p) return "null params";
    if (p->max_batch < 1 || p->max_batch > 1024) return "max_batch out of range";
    if (p->max_k < 1 || p->max_k > 32) return "max_k must be in 1..32";
    if (p->max_seq < 64 || p->max_seq % 64) return "max_seq must be a positive multiple of 64";
    if (const char *e = check_model(p->target)) return e;
    if (const char *e = check_model(p->drafter)) return e;
    if (p->target.vocab != p->drafter.vocab) return "target and drafter must share the vocabulary";
    if (p->mask_token_id < 0 || p->mask_token_id >= p->drafter.vocab) return "mask_token_id outside the vocabulary";
    if (p->eos_token_id >= p->target.vocab) return "eos_token_id outside the vocabulary";
    return nullptr;
}

// ---------------------------------------------------------------------------------------------
// launches
// ---------------------------------------------------------------------------------------------
// K splits per column group: as many as keep the launch within one wave of workgroups (rounded down: a second
// wave of workgroups costs more than idle CUs).  Measured on MI355X with the 8B- and 4B-shaped matrices: the split-K
// tail (partial store, arrival, the last workgroup's sum) makes ~224 workgroups the best target for matrices with up
// to 256 k-steps, 256 for longer contractions; at most 8 splits; none for contractions of up to 64 k-steps.
int choose_split(int N, int KS, int zgroups) {
    const int blocks = (N / CG) * zgroups;
    const int target = KS > 256 ? 256 : 224;
    int S = std::max(1, target / blocks);
    // the workgroup that finishes a column group sums S partial tiles (about 0.25 us each) before its epilogue:
    // beyond 8 splits that costs more than the shorter streams save (drafter down projection, 7 column groups:
    // 19 splits 22.8 us, 8 splits 18.5 us)
    S = std::min(S, 8);
    // a short contraction (the drafter's d = 896: 56 k-steps) is not split at all: the partial store, the arrival
    // and the last workgroup's sum cost more than streaming a 128-column slab from one workgroup (2.44 -> 2.36 ms per draft pass)
    if (KS <= 64) S = 1;
    S = std::min(S, std::max(1, KS / 16));           // at least 16 k-steps per workgroup
    S = std::min<int>(S, (int)(PART_COLS / (size_t)N));
    return std::max(S, 1);
}

// deer_debug_gemm_stamps: the chosen launch and the one after it record their workgroups' stamps, each in its half of
// the buffer (zeroed at the start of the pass); null for every other launch or one with too many workgroups.
unsigned long long *stamp_buffer(deer_ctx *c, size_t workgroups) {
    const int stamp_rel = c->gemm_launch_idx - c->stamp_launch;
    if (c->stamp_launch < 0 || c->cur_pass_model != c->stamp_model || (stamp_rel != 0 && stamp_rel != 1) ||
        workgroups > (size_t)STAMP_MAX_BLOCKS / 2)
        return nullptr;
    c->stamp_blocks = STAMP_MAX_BLOCKS;
    return c->wk.stamps + (size_t)stamp_rel * (STAMP_MAX_BLOCKS / 2) * 8;
}

template <int EPI>
int launch_gemm(deer_ctx *c, GemmArgs &a, int K, int ntiles, int force_S) {
    a.KS = K / 16;
    // Row tiles go through a workgroup in pairs (the weights are read once per pair) unless the matrix is small:
    // then every tile gets workgroups of its own, which find the weights in their XCD's L2, and the workgroup that
    // finishes a column group runs one epilogue instead of two in a row.  Measured on MI355X: the 0.5B drafter's
    // pass over two row tiles 2.26 -> 1.71 ms, over 16 tiles (batch 8) 3.73 -> 3.39 ms, over 32 tiles 5.56 -> 5.80 ms
    // (pairs stay); of the 8B shape's matrices the 33.6 MB output projection gains up to 8 tiles and the 50.3 MB QKV
    // projection up to 4 (batch 2 verify 5.99 -> 5.82 ms), gate/up and down lose at any tile count.
    constexpr double mt1_bytes = 5.1e7, mt1_product = 2.8e8;
    constexpr int mt1_tiles = 16;
    // (matrix bytes x tiles is capped too: the output projection loses at 16 tiles)
    const double w_bytes = (double)a.N * K * 2.0;
    const bool pairs = ntiles % 2 == 0 && !(ntiles <= mt1_tiles && w_bytes <= mt1_bytes && w_bytes * ntiles <= mt1_product);
    const int MT = pairs ? 2 : 1;
    const int zg = ntiles / MT;
    a.rows_total = ntiles * 32;
    {   // many rows and enough 256 x 256 tiles to fill the chip: blocked for the matrix cores
        const int ncg = a.N / CG;
        const int tiles = ((ntiles + TG_RT - 1) / TG_RT) * ((ncg + 1) / 2);
        // measured: at 512 and 1024 rows (two and four row blocks) the streaming kernel with shared L2 lines is still
        // ahead (config-5 verify 41.9 against 47.7 ms); from 1024 rows on the blocked kernel wins where it has 128 tiles
        // (prefill 133 against 167 ms; two 512-token sequences recomputed per iteration 44.3 against 46.8 ms)
        constexpr int rows_tiles = 32;
        const int min_rows_tiles = c->tiled_min_tiles >= 128 ? rows_tiles : TG_RT;   // tests lower both thresholds
        if (c->tiled_min_tiles > 0 && EPI != EPI_ROUTER && ntiles >= min_rows_tiles && a.KS % TG_KST == 0 && tiles >= c->tiled_min_tiles) {
            a.S = 1; a.part = nullptr; a.counters = nullptr;
            ProfScope ps(c, 0, (double)a.N * K * 2.0);
            hipLaunchKernelGGL((k_gemm_tiled<EPI>), dim3((unsigned)tiled_blocks(ntiles, ncg)), dim3(512), 0, c->stream, a, ncg, ntiles);
            LAUNCHCHK(c, "k_gemm_tiled");
            return DEER_OK;
        }
    }
    if ((EPI == EPI_RESID || (EPI == EPI_QKV && a.hd <= 64 && 64 % a.hd == 0 && a.N % 64 == 0)) && a.ssq_sub == 4 && MT == 1 &&
        force_S <= 0 && a.KS <= 64) {
        // an unsplit GEMM of a small model: one workgroup per row tile and 32-column weight block (residual GEMM) or
        // 64-column pair of blocks (QKV: whole heads)
        a.S = 1; a.part = nullptr; a.counters = nullptr;
        const int ngrp = EPI == EPI_RESID ? a.N / 32 : a.N / 64;
        a.stamps = stamp_buffer(c, (size_t)ngrp * ntiles);
        c->gemm_launch_idx++;
        ProfScope ps(c, 0, (double)a.N * K * 2.0);
        const dim3 g1((unsigned)(((ngrp + 7) / 8) * 8 * ntiles));
        if (EPI == EPI_RESID) hipLaunchKernelGGL((k_gemm_narrow<1, EPI_RESID>), g1, dim3(512), 0, c->stream, a, ngrp, ntiles);
        else hipLaunchKernelGGL((k_gemm_narrow<2, EPI_QKV>), g1, dim3(512), 0, c->stream, a, ngrp, ntiles);
        LAUNCHCHK(c, "k_gemm_narrow");
        return DEER_OK;
    }
    a.S = force_S > 0 ? force_S : choose_split(a.N, a.KS, zg);
    while (a.S > 1 && (size_t)a.S * a.rows_total * a.N > c->wk.part_floats) --a.S;   // partials must fit their buffer
    a.part = (EPI == EPI_LMHEAD) ? nullptr : c->wk.part;
    a.counters = c->wk.gemm_cnt;
    a.stamps = stamp_buffer(c, (size_t)(a.N / CG) * a.S * zg);
    c->gemm_launch_idx++;
    dim3 grid(a.N / CG, a.S, zg);
    ProfScope ps(c, 0, (double)a.N * K * 2.0);
    if (zg > 1) {   // the row-tile groups of a (column group, K split) pair share an XCD's L2
        const int ncg = a.N / CG, pairs8 = (ncg * a.S + 7) / 8;
        dim3 g1((unsigned)(pairs8 * 8 * zg));
        if (MT == 2) hipLaunchKernelGGL((k_gemm_rows<2, EPI>), g1, dim3(512), 0, c->stream, a, ncg, zg);
        else hipLaunchKernelGGL((k_gemm_rows<1, EPI>), g1, dim3(512), 0, c->stream, a, ncg, zg);
    } else if (MT == 2) hipLaunchKernelGGL((k_gemm<2, EPI>), grid, dim3(512), 0, c->stream, a);
    else hipLaunchKernelGGL((k_gemm<1, EPI>), grid, dim3(512), 0, c->stream, a);
    LAUNCHCHK(c, "k_gemm");
    return DEER_OK;
}

// draw: the pass samples its rows' tokens (Gumbel-max over the perturbed logits): the drafter's pass at T > 0; the target's
// rows only need the maximum and the sum of exponentials
struct LmPlan { bool on; int mt0, mt_stride, n_tiles, k; float T; uint64_t seed; int k_lo = 0; bool draw = false; };

template <int HD>
int launch_attn(deer_ctx *c, ModelRT &m, int layer, int ntiles, int NS, int NS_head, float scale_log2e, double kv_bytes,
                const NextWeights &nx) {
    Work &w = c->wk;
    const deer_model_cfg &mc = m.c;
    const uint16_t *K = m.kv + m.kv_k_base + (size_t)layer * m.kv_layer_stride;
    const uint16_t *Vt = m.kv + m.kv_v_base + (size_t)layer * m.kv_layer_stride;
    ProfScope ps(c, 1, kv_bytes);
    if (NS_head > 0) {   // few tiles: one workgroup per (tile, query head, key range), merged by the last to arrive
        hipLaunchKernelGGL(k_attn_head<HD>, dim3(mc.n_q_heads * NS_head, ntiles), dim3(512), 0, c->stream, w.q_hi, w.q_lo, K, Vt,
                           m.kv_seq_stride, m.kv_head_stride, w.rm.tile_seq, w.rm.limit, w.opart, w.attn_cnt,
                           mc.n_q_heads, mc.n_kv_heads, NS_head, scale_log2e, w.xb_hi, w.xb_lo, nx);
        LAUNCHCHK(c, "k_attn_head");
        return DEER_OK;
    }
    hipLaunchKernelGGL(k_attn<HD>, dim3(mc.n_kv_heads * NS, ntiles), dim3(512), 0, c->stream, w.q_hi, w.q_lo, K, Vt,
                       m.kv_seq_stride, m.kv_head_stride, c->p.max_seq, w.rm.tile_seq, w.rm.limit, w.opart,
                       mc.n_q_heads, mc.n_kv_heads, NS, scale_log2e, w.xb_hi, w.xb_lo);
    LAUNCHCHK(c, "k_attn");
    if (NS > 1) {
        const int n_items = ntiles * mc.n_q_heads * (HD / 32) * 2;
        hipLaunchKernelGGL(k_attn_merge<HD>, dim3((n_items + 3) / 4), dim3(256), 0, c->stream, w.opart, NS, mc.n_q_heads, n_items,
                           scale_log2e, w.xb_hi, w.xb_lo);
        LAUNCHCHK(c, "k_attn_merge");
    }
    return DEER_OK;
}

// One forward pass of `model` over the rows described by the row metadata (ntiles tiles).
// rows: the pass's rows are described by a PassRows (draft, verify): one launch works them out, gathers the embeddings
// and fills the RoPE table; null: the row metadata is in place already (prefill).
int run_pass(deer_ctx *c, int model, int ntiles, int max_limit, const LmPlan &lm, double kv_keys_total = 0.0,
             const PassRows *rows_desc = nullptr) {
    ModelRT &m = c->m[model];
    Work &w = c->wk;
    const deer_model_cfg &mc = m.c;
    const int d = mc.d_model, hd = mc.head_dim, rows = ntiles * 32, ncg_d = d / CG;
    c->gemm_launch_idx = 0;
    c->cur_pass_model = model;
    hipStream_t s = c->stream;
    if (c->stamp_launch >= 0 && model == c->stamp_model) (void)hipMemsetAsync(w.stamps, 0, (size_t)STAMP_MAX_BLOCKS * 64, s);
    prof_close(c);
    if (rows_desc) {
        hipLaunchKernelGGL(k_pass_begin, dim3(ncg_d + 1, ntiles), dim3(256), 0, s, *rows_desc, w.rm, (const uint16_t *)(m.w + m.off_embed),
                           w.h, w.xa_hi, w.xa_lo, w.ssq, d, ncg_d, m.ssq_sub, m.theta, w.cs, hd / 2);
        LAUNCHCHK(c, "k_pass_begin");
    } else {
        hipLaunchKernelGGL(k_embed, dim3(ncg_d, ntiles), dim3(256), 0, s, (const uint16_t *)(m.w + m.off_embed), w.rm.tok, w.h,
                           w.xa_hi, w.xa_lo, w.ssq, d, ncg_d, m.ssq_sub);
        LAUNCHCHK(c, "k_embed");
        int n = rows * (hd / 2);
        hipLaunchKernelGGL(k_rope_table, dim3((n + 255) / 256), dim3(256), 0, s, w.rm.pos, m.theta, w.cs, hd / 2, rows);
        LAUNCHCHK(c, "k_rope_table");
    }
    const int nkt = (max_limit + 31) / 32;
    // key-range splits: aim at one workgroup per compute unit; a split holds at least one staged chunk of 4 key
    // tiles; ntiles * NS never exceeds the partial buffer (max(64, most tiles of a pass) tile slots)
    constexpr int ns_target = 256;
    int NS = (ns_target + mc.n_kv_heads * ntiles - 1) / (mc.n_kv_heads * ntiles);
    NS = std::max(1, std::min({NS, MAX_NS, std::max(1, std::max(64, c->max_tiles) / ntiles), (nkt + 3) / 4}));
    // Passes of few tiles (decoding) run attention per query head: (tile, head, key range) workgroups, about one per
    // compute unit, as long as a wave then has at most ATT_HEAD_MAX_TILES key tiles of its range to go through
    int NS_head = 0;
    if (ntiles * mc.n_q_heads <= ns_target) {
        int ns = ns_target / (ntiles * mc.n_q_heads);
        ns = std::max(1, std::min({ns, MAX_NS, std::max(1, std::max(64, c->max_tiles) / ntiles), (nkt + 7) / 8}));
        const int per = (nkt + ns - 1) / ns;
        if ((per + 7) / 8 <= ATT_HEAD_MAX_TILES) NS_head = ns;
    }
    const float scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)hd));
    const double kv_bytes = kv_keys_total * mc.n_kv_heads * hd * 2.0 * 2.0;   // K and V rows read per layer
    GemmArgs base{};
    base.mt0 = 0; base.mt_stride = 1;
    base.ssq_in = w.ssq; base.ncg_in = ncg_d * m.ssq_sub; base.d_in = d; base.eps = mc.rms_eps;
    base.ssq_sub = m.ssq_sub;
    base.cs = w.cs; base.rm = w.rm; base.qhi = w.q_hi; base.qlo = w.q_lo;
    base.Hq = mc.n_q_heads; base.Hkv = mc.n_kv_heads; base.hd = hd;
    base.h = w.h; base.xhi_out = w.xa_hi; base.xlo_out = w.xa_lo; base.ssq_out = w.ssq;
    base.ahi = w.xb_hi; base.alo = w.xb_lo; base.F = m.F;
    // What the idle workgroups of a split launch pull into their XCD's L2 for the launch after it (passes of one row
    // tile, wide workgroups): the first k-steps of every workgroup of the next GEMM — attention fetches for the output
    // projection, the down projection for the next layer's QKV projection — and, from the QKV projection, the old K,V
    // blocks of the kv head its XCD serves in the per-head attention launch.  Measured (8B target, prefix 4096): verify
    // pass 4.29 -> 4.21 ms; more than 16 KB per 32-column block, or fetching from unsplit launches (after their
    // epilogue) or for gate/up, costs more than it saves.
    // A small dense model (narrow workgroups for its unsplit O and QKV projections, one or two row tiles): attention
    // fetches the output projection's 32-column blocks whole, the split down projection the next layer's QKV blocks.
    const bool fetch_ahead = ntiles == 1 && m.ssq_sub == 1;
    const bool fetch_ahead_narrow = ntiles <= 2 && m.ssq_sub == 4 && !mc.n_experts;
    auto next_plan_narrow = [&](const char *W, int N, int K, int NB) {   // NB: 1 residual GEMM, 2 QKV (whole heads)
        NextWeights nx{};
        const int KS = K / 16;
        if (!fetch_ahead_narrow || KS > 64 || N % (32 * NB)) return nx;
        if (NB == 2 && !(hd <= 64 && 64 % hd == 0)) return nx;
        nx.base = W; nx.ncg = N / (32 * NB); nx.nwg = ((nx.ncg + 7) / 8) * 8 * ntiles;
        nx.block_bytes = (long long)KS * 1024; nx.narrow_nb = NB; nx.Z = ntiles;
        return nx;
    };
    auto next_plan = [&](const char *W, int N, int K) {
        NextWeights nx{};
        if (!fetch_ahead) return nx;
        const int KS = K / 16;
        int S = choose_split(N, KS, 1);
        while (S > 1 && (size_t)S * 32 * N > c->wk.part_floats) --S;
        const int per = (KS + S * 8 - 1) / (S * 8);
        nx.base = W; nx.ncg = N / CG; nx.nwg = nx.ncg * S; nx.span = NEXT_SPAN_BYTES;
        nx.block_bytes = (long long)KS * 1024; nx.split_bytes = (long long)8 * per * 1024;
        return nx;
    };
    for (int l = 0; l < mc.n_layers; ++l) {
        const char *lw = m.w + m.off_layers + (size_t)l * m.layer_bytes;
        GemmArgs a = base;
        a.W = (const uint4 *)(lw + m.lo_qkv); a.Xhi = w.xa_hi; a.Xlo = w.xa_lo; a.N = m.n_qkv;
        a.kv = KvView{m.kv + m.kv_k_base + (size_t)l * m.kv_layer_stride, m.kv + m.kv_v_base + (size_t)l * m.kv_layer_stride,
                      m.kv_seq_stride, m.kv_head_stride, c->p.max_seq};
        // whole key tiles that no row of this pass writes (a pass of one tile appends at most 32 rows)
        if (fetch_ahead && NS_head > 0 && c->batch == 1 && 8 % mc.n_kv_heads == 0)
            a.kv_fetch_bytes = std::min(KV_FETCH_MAX_BYTES, std::max(0, (max_limit - 32) / 32) * 32 * hd * 2);
        int rc = launch_gemm<EPI_QKV>(c, a, d, ntiles, 0);
        if (rc) return rc;
        const NextWeights nx_o = fetch_ahead_narrow ? next_plan_narrow(lw + m.lo_o, d, m.kattn, 1) : next_plan(lw + m.lo_o, d, m.kattn);
        if (hd == 128) rc = launch_attn<128>(c, m, l, ntiles, NS, NS_head, scale_log2e, kv_bytes, nx_o);
        else if (hd == 64) rc = launch_attn<64>(c, m, l, ntiles, NS, NS_head, scale_log2e, kv_bytes, nx_o);
        else rc = launch_attn<32>(c, m, l, ntiles, NS, NS_head, scale_log2e, kv_bytes, nx_o);
        if (rc) return rc;
        a = base;
        a.W = (const uint4 *)(lw + m.lo_o); a.Xhi = w.xb_hi; a.Xlo = w.xb_lo; a.N = d;
        rc = launch_gemm<EPI_RESID>(c, a, m.kattn, ntiles, 0);
        if (rc) return rc;
        if (!mc.n_experts) {
            a = base;
            a.W = (const uint4 *)(lw + m.lo_gu); a.Xhi = w.xa_hi; a.Xlo = w.xa_lo; a.N = 2 * m.F;
            rc = launch_gemm<EPI_SWIGLU>(c, a, d, ntiles, 0);
            if (rc) return rc;
            a = base;
            a.W = (const uint4 *)(lw + m.lo_d); a.Xhi = w.xb_hi; a.Xlo = w.xb_lo; a.N = d;
            if (l + 1 < mc.n_layers)
                a.nx = fetch_ahead_narrow ? next_plan_narrow(lw + m.layer_bytes + m.lo_qkv, m.n_qkv, d, 2)
                                          : next_plan(lw + m.layer_bytes + m.lo_qkv, m.n_qkv, d);
            rc = launch_gemm<EPI_RESID>(c, a, m.F, ntiles, 0);
            if (rc) return rc;
        } else {
            // router -> per-expert grouping -> grouped gate/up and down GEMMs -> ordered combine
            a = base;
            a.W = (const uint4 *)(lw + m.lo_router); a.Xhi = w.xa_hi; a.Xlo = w.xa_lo; a.N = CG;
            a.n_experts = mc.n_experts; a.top_k = mc.top_k; a.route_e = w.route_e; a.route_w = w.route_w;
            a.route_spread = (c->route_spread && (mc.n_experts & (mc.n_experts - 1)) == 0) ? l + 1 : 0;
            rc = launch_gemm<EPI_ROUTER>(c, a, d, ntiles, 0);
            if (rc) return rc;
            const int cap = rows, chunks = ntiles;
            prof_close(c);
            hipLaunchKernelGGL(k_moe_group, dim3(1), dim3(256), 0, s, w.route_e, w.rm.slot, rows, mc.top_k, mc.n_experts, cap,
                               w.exp_cnt, w.pair_row, w.pair_slot, w.moe_touched);
            LAUNCHCHK(c, "k_moe_group");
            MoeArgs ma{};
            ma.cap = cap; ma.chunks = chunks; ma.cnt = w.exp_cnt; ma.pair_row = w.pair_row; ma.pair_slot = w.pair_slot;
            ma.ssq_in = w.ssq; ma.ncg_in = ncg_d; ma.d_in = d; ma.eps = mc.rms_eps;
            ma.ahi = w.act_hi; ma.alo = w.act_lo; ma.Fe = m.F; ma.route_w = w.route_w; ma.moe_out = w.moe_out; ma.d = d;
            ma.W = (const uint4 *)(lw + m.lo_gu); ma.wexp_stride = m.exp_gu_bytes / 16; ma.Xhi = w.xa_hi; ma.Xlo = w.xa_lo;
            ma.N = 2 * m.F; ma.KS = d / 16;
            {
                ProfScope ps(c, 0, 0.0);
                hipLaunchKernelGGL(k_gemm_moe<MOE_GATEUP>, dim3((2 * m.F / CG + MOE_CGS - 1) / MOE_CGS, mc.n_experts, chunks), dim3(512), 0, s, ma);
            }
            LAUNCHCHK(c, "k_gemm_moe gate/up");
            ma.W = (const uint4 *)(lw + m.lo_d); ma.wexp_stride = m.exp_d_bytes / 16; ma.Xhi = w.act_hi; ma.Xlo = w.act_lo;
            ma.N = d; ma.KS = m.F / 16;
            {
                ProfScope ps(c, 0, 0.0);
                hipLaunchKernelGGL(k_gemm_moe<MOE_DOWN>, dim3((d / CG + MOE_CGS - 1) / MOE_CGS, mc.n_experts, chunks), dim3(512), 0, s, ma);
            }
            LAUNCHCHK(c, "k_gemm_moe down");
            prof_close(c);
            hipLaunchKernelGGL(k_moe_combine, dim3(ncg_d, ntiles), dim3(256), 0, s, w.moe_out, w.rm.slot, mc.top_k, w.h, w.xa_hi,
                               w.xa_lo, w.ssq, d);
            LAUNCHCHK(c, "k_moe_combine");
        }
    }
    if (lm.on) {
        const int V = mc.vocab;
        GemmArgs a = base;
        a.W = (const uint4 *)(m.w + m.off_lm); a.Xhi = w.xa_hi; a.Xlo = w.xa_lo; a.N = V;
        a.mt0 = lm.mt0; a.mt_stride = lm.mt_stride;
        a.k = lm.k; a.k_lo = lm.k_lo; a.T = lm.T; a.seed = lm.seed; a.draw = lm.draw ? 1 : 0; a.stat = w.stat; a.ncg_v = V / CG;
        a.logits = (c->p.keep_logits || lm.T > 0.f) ? w.logits[model] : nullptr;
        int rc = launch_gemm<EPI_LMHEAD>(c, a, d, lm.n_tiles, 1);
        if (rc) return rc;
        prof_close(c);
        hipLaunchKernelGGL(k_rowstat_final, dim3(lm.n_tiles * lm.k), dim3(256), 0, s, w.stat, V / CG, lm.T, w.res[model], lm.k, lm.k_lo);
        LAUNCHCHK(c, "k_rowstat_final");
    }
    prof_close(c);
    return DEER_OK;
}

int upload_state(deer_ctx *c, int B, const int *len, const int *dr_len, const int *pending) {
    Work &w = c->wk;
    std::vector<int> zeros(B, 0);
    HIPCHK(c, hipMemcpyAsync(w.st.len, len, B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(w.st.dr_len, dr_len, B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(w.st.pending, pending, B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(w.st.ing_n, zeros.data(), B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(w.st.finished, zeros.data(), B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->batch = B;
    c->h_len.assign(len, len + B);
    c->h_ing_n.assign(B, 0);
    c->h_finished.assign(B, 0);
    c->state = ST_PREFILLED;
    return DEER_OK;
}

}  // namespace

// =============================================================================================
// C ABI
// =============================================================================================
extern "C" {

int deer_query_sizes(const deer_init_params *p, deer_sizes *out) {
    if (!out) return fail(nullptr, DEER_EINVAL, "null output");
    if (p && (p->struct_size != sizeof(deer_init_params) || p->abi_version != DEER_ABI_VERSION))
        return fail(nullptr, DEER_EVERSION, "struct_size/abi_version mismatch");
    if (const char *e = check_params(p)) return fail(nullptr, DEER_EINVAL, "%s", e);
    ModelRT m;
    for (int i = 0; i < 2; ++i) {
        plan_model(m, i == 0 ? p->target : p->drafter, p->max_batch, p->max_seq);
        out->weights[i] = m.weight_bytes;
        out->kv[i] = m.kv_bytes;
    }
    Work w;
    plan_work(w, *p, nullptr);
    out->workspace = w.bytes;
    out->staging = 0;
    return DEER_OK;
}

int deer_init_models(const deer_init_params *p, const deer_buffers *bufs, const deer_sizes *buf_sizes, deer_ctx **out) {
    if (out) *out = nullptr;
    if (!out || !bufs || !buf_sizes) return fail(nullptr, DEER_EINVAL, "null argument");
    deer_sizes need;
    int rc = deer_query_sizes(p, &need);
    if (rc) return rc;
    for (int i = 0; i < 2; ++i) {
        if (!bufs->weights[i] || !bufs->kv[i]) return fail(nullptr, DEER_EINVAL, "null device buffer");
        if (buf_sizes->weights[i] < need.weights[i] || buf_sizes->kv[i] < need.kv[i])
            return fail(nullptr, DEER_ECAPACITY, "weights/kv buffer %d too small", i);
    }
    if (!bufs->workspace) return fail(nullptr, DEER_EINVAL, "null workspace");
    if (buf_sizes->workspace < need.workspace) return fail(nullptr, DEER_ECAPACITY, "workspace too small");
    deer_ctx *c = new (std::nothrow) deer_ctx();
    if (!c) return fail(nullptr, DEER_EINVAL, "out of host memory");
    c->p = *p;
    c->stream = (hipStream_t)p->hip_stream;
    hipError_t e = hipSetDevice(p->device);
    if (e != hipSuccess) { delete c; return fail(nullptr, DEER_EHIP, "hipSetDevice: %s", hipGetErrorString(e)); }
    if (p->device >= 0 && p->device < MAX_DEVICES) {   // this device's address of the static scratch array
        if (!g_scratch_ptr[p->device]) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess) { delete c; return fail(nullptr, DEER_EHIP, "hipGetSymbolAddress: %s", hipGetErrorString(e)); }
            g_scratch_ptr[p->device] = ptr;
        }
        c->static_scratch = g_scratch_ptr[p->device];
    }
    for (int i = 0; i < 2; ++i) {
        plan_model(c->m[i], i == 0 ? p->target : p->drafter, p->max_batch, p->max_seq);
        c->m[i].w = (char *)bufs->weights[i];
        c->m[i].kv = (uint16_t *)bufs->kv[i];
    }
    plan_work(c->wk, *p, (char *)bufs->workspace);
    c->max_tiles = std::max(2 * p->max_batch, prefill_tiles(*p));
    // caches must hold finite values everywhere: masked keys are multiplied by zero weights
    for (int i = 0; i < 2; ++i) {
        e = hipMemsetAsync(bufs->kv[i], 0, need.kv[i], c->stream);
        if (e != hipSuccess) { delete c; return fail(nullptr, DEER_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); }
        const deer_model_cfg &mc = c->m[i].c;
        double th[64];
        for (int k = 0; k < mc.head_dim / 2; ++k) th[k] = std::pow((double)mc.rope_base, -2.0 * k / mc.head_dim);
        c->m[i].theta = c->wk.theta[i];
        e = hipMemcpy(c->m[i].theta, th, sizeof(double) * (mc.head_dim / 2), hipMemcpyHostToDevice);
        if (e != hipSuccess) { delete c; return fail(nullptr, DEER_EHIP, "hipMemcpy: %s", hipGetErrorString(e)); }
    }
    if (c->wk.moe_touched) (void)hipMemsetAsync(c->wk.moe_touched, 0, 8, c->stream);
    e = hipMemsetAsync(c->wk.cnt_base, 0, c->wk.cnt_bytes, c->stream);
    if (e != hipSuccess) { delete c; return fail(nullptr, DEER_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); }
    e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) { delete c; return fail(nullptr, DEER_EHIP, "hipStreamSynchronize: %s", hipGetErrorString(e)); }
    {   // a few KB of page-locked host memory for the acceptance results (host memory: the device buffers stay the caller's)
        const size_t bytes = (size_t)((const char *)c->wk.ao.committed - (const char *)c->wk.ao.accept_len) + (size_t)p->max_batch * 32 * 4;
        void *hp = nullptr;
        if (hipHostMalloc(&hp, bytes, hipHostMallocDefault) == hipSuccess) { c->h_pin = (char *)hp; c->h_pin_bytes = bytes; }
        else (void)hipGetLastError();
    }
    *out = c;
    return DEER_OK;
}

int deer_load_tensor(deer_ctx *c, int model, int tensor_id, int layer, int expert, const void *src, int src_dtype,
                     int64_t rows, int64_t cols) {
    if (!c) return DEER_EINVAL;
    if (!src || model < 0 || model > 1 || (src_dtype != DEER_F32 && src_dtype != DEER_BF16))
        return fail(c, DEER_EINVAL, "bad model/dtype/pointer");
    ModelRT &m = c->m[model];
    const deer_model_cfg &mc = m.c;
    const int d = mc.d_model, hd = mc.head_dim;
    int64_t er = 0, ec = 0;
    char *dst = nullptr;
    int mode = 0, col_off = 0, K = 0;
    const bool per_layer = tensor_id >= DEER_T_WQ && tensor_id <= DEER_T_ROUTER;
    const bool per_expert = mc.n_experts && (tensor_id == DEER_T_WG || tensor_id == DEER_T_WU || tensor_id == DEER_T_WD);
    if (per_expert && (expert < 0 || expert >= mc.n_experts)) return fail(c, DEER_EINVAL, "expert out of range");
    if (!per_expert && expert >= 0) return fail(c, DEER_EINVAL, "tensor %d takes no expert index", tensor_id);
    const size_t ex = per_expert ? (size_t)expert : 0;
    if (per_layer && (layer < 0 || layer >= mc.n_layers)) return fail(c, DEER_EINVAL, "layer out of range");
    char *lw = m.w + m.off_layers + (size_t)(per_layer ? layer : 0) * m.layer_bytes;
    switch (tensor_id) {
        case DEER_T_EMBED: er = mc.vocab; ec = d; dst = m.w + m.off_embed; break;
        case DEER_T_LM_HEAD: er = d; ec = mc.vocab; dst = m.w + m.off_lm; K = d; break;
        case DEER_T_WQ: er = d; ec = mc.n_q_heads * hd; dst = lw + m.lo_qkv; K = d; break;
        case DEER_T_WK: er = d; ec = mc.n_kv_heads * hd; dst = lw + m.lo_qkv; K = d; col_off = mc.n_q_heads * hd; break;
        case DEER_T_WV: er = d; ec = mc.n_kv_heads * hd; dst = lw + m.lo_qkv; K = d; col_off = (mc.n_q_heads + mc.n_kv_heads) * hd; break;
        case DEER_T_WO: er = m.kattn; ec = d; dst = lw + m.lo_o; K = m.kattn; break;
        case DEER_T_WG: er = d; ec = m.F; dst = lw + m.lo_gu + ex * m.exp_gu_bytes; K = d; mode = 1; break;
        case DEER_T_WU: er = d; ec = m.F; dst = lw + m.lo_gu + ex * m.exp_gu_bytes; K = d; mode = 2; break;
        case DEER_T_WD: er = m.F; ec = d; dst = lw + m.lo_d + ex * m.exp_d_bytes; K = m.F; break;
        case DEER_T_ROUTER:
            if (!mc.n_experts) return fail(c, DEER_EINVAL, "model has no router");
            er = d; ec = mc.n_experts; dst = lw + m.lo_router; K = d; break;
        default: return fail(c, DEER_EINVAL, "unknown tensor id %d", tensor_id);
    }
    if (rows != er || cols != ec) return fail(c, DEER_EINVAL, "tensor %d: expected %lld x %lld, got %lld x %lld", tensor_id,
                                              (long long)er, (long long)ec, (long long)rows, (long long)cols);
    if (tensor_id == DEER_T_EMBED) {
        size_t n = (size_t)rows * cols;
        dim3 grid((unsigned)((n + 255) / 256));
        if (src_dtype == DEER_F32) hipLaunchKernelGGL(k_convert_rows<float>, grid, dim3(256), 0, c->stream, (const float *)src, (uint16_t *)dst, n);
        else hipLaunchKernelGGL(k_convert_rows<uint16_t>, grid, dim3(256), 0, c->stream, (const uint16_t *)src, (uint16_t *)dst, n);
    } else {
        size_t n = (size_t)(K / 8) * cols;
        dim3 grid((unsigned)((n + 255) / 256));
        if (src_dtype == DEER_F32) hipLaunchKernelGGL(k_repack<float>, grid, dim3(256), 0, c->stream, (const float *)src, (uint4 *)dst, K, (int)cols, K / 16, mode, col_off);
        else hipLaunchKernelGGL(k_repack<uint16_t>, grid, dim3(256), 0, c->stream, (const uint16_t *)src, (uint4 *)dst, K, (int)cols, K / 16, mode, col_off);
    }
    LAUNCHCHK(c, "k_repack");
    return DEER_OK;
}

int deer_prefill(deer_ctx *c, int32_t batch, const int32_t *ids, const int32_t *lens) {
    if (!c) return DEER_EINVAL;
    if (!ids || !lens || batch < 1 || batch > c->p.max_batch) return fail(c, DEER_EINVAL, "bad batch or null pointer");
    for (int b = 0; b < batch; ++b) {
        if (lens[b] < 1) return fail(c, DEER_EINVAL, "prompt %d is empty", b);
        if (lens[b] + c->p.max_k > c->p.max_seq) return fail(c, DEER_ECAPACITY, "prompt %d: %d tokens + one block exceed max_seq %d", b, lens[b], c->p.max_seq);
    }
    Work &w = c->wk;
    std::vector<int> pend(batch), lenv(lens, lens + batch);
    std::vector<size_t> offs(batch);
    size_t total = 0;
    for (int b = 0; b < batch; ++b) {
        offs[b] = total;
        for (int i = 0; i < lens[b]; ++i)
            if (ids[total + i] < 0 || ids[total + i] >= c->p.target.vocab) return fail(c, DEER_EINVAL, "token id outside the vocabulary");
        total += lens[b];
        pend[b] = ids[total - 1];
    }
    HIPCHK(c, hipMemcpyAsync(w.ids, ids, total * 4, hipMemcpyHostToDevice, c->stream));
    // Passes of up to cap tiles; a pass takes the next rows of as many sequences as fit, each sequence's rows in
    // whole tiles (rows of one sequence that are split over passes continue in the next pass, over the keys the
    // earlier pass has written).  The descriptor lists stay alive until the stream has been waited for.
    const int cap = prefill_tiles(c->p);
    std::vector<std::vector<int4>> kept;
    for (int model = 0; model < 2; ++model) {
        std::vector<int4> desc;
        int maxlim = 0;
        auto flush = [&]() -> int {
            if (desc.empty()) return DEER_OK;
            kept.push_back(desc);
            const std::vector<int4> &dsc = kept.back();
            const int ntiles = (int)dsc.size();
            HIPCHK(c, hipMemcpyAsync(w.pf_desc, dsc.data(), dsc.size() * sizeof(int4), hipMemcpyHostToDevice, c->stream));
            hipLaunchKernelGGL(k_rows_prefill, dim3(ntiles), dim3(32), 0, c->stream, w.rm, w.ids, w.pf_desc);
            LAUNCHCHK(c, "k_rows_prefill");
            LmPlan lm{false, 0, 1, 0, 0, 0.f, 0};
            int rc = run_pass(c, model, ntiles, maxlim, lm);
            desc.clear();
            maxlim = 0;
            return rc;
        };
        for (int b = 0; b < batch; ++b) {
            const int nrows = (model == DEER_TARGET) ? lens[b] - 1 : lens[b];   // the last token stays pending for the target
            int c0 = 0;
            while (c0 < nrows) {
                if ((int)desc.size() == cap)
                    if (int rc = flush()) return rc;
                const int room = cap - (int)desc.size();
                const int take = std::min(nrows - c0, room * 32);
                for (int i = 0; i < take; i += 32)
                    desc.push_back(make_int4(b, c0 + i, std::min(32, take - i), (int)(offs[b] + c0 + i)));
                maxlim = std::max(maxlim, c0 + take);
                c0 += take;
            }
        }
        if (int rc = flush()) return rc;
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return upload_state(c, batch, lenv.data(), lenv.data(), pend.data());
}

int deer_set_prefilled(deer_ctx *c, int32_t batch, const int32_t *lens, const int32_t *last) {
    if (!c) return DEER_EINVAL;
    if (!lens || !last || batch < 1 || batch > c->p.max_batch) return fail(c, DEER_EINVAL, "bad batch or null pointer");
    for (int b = 0; b < batch; ++b) {
        if (lens[b] < 1) return fail(c, DEER_EINVAL, "sequence %d is empty", b);
        if (lens[b] + c->p.max_k > c->p.max_seq) return fail(c, DEER_ECAPACITY, "sequence %d exceeds max_seq", b);
        if (last[b] < 0 || last[b] >= c->p.target.vocab) return fail(c, DEER_EINVAL, "token id outside the vocabulary");
    }
    return upload_state(c, batch, lens, lens, last);
}

int deer_draft_block_multipass(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t n_passes, int32_t *draft_dev) {
    if (!c) return DEER_EINVAL;
    if (!draft_dev || k < 1 || k > c->p.max_k || !(T >= 0.f)) return fail(c, DEER_EINVAL, "bad k, T or null pointer");
    if (n_passes < 1 || n_passes > k) return fail(c, DEER_EINVAL, "n_passes must be in 1..k");
    if (c->state != ST_PREFILLED) return fail(c, DEER_ESTATE, "draft_block needs a prefilled or committed state");
    if (k + c->bonus > 32) return fail(c, DEER_EINVAL, "with the bonus token on, k must be at most 31 (k + 1 rows per tile)");
    const int B = c->batch;
    int maxlim = 0, any_ing = 0;
    for (int b = 0; b < B; ++b) {
        if (c->h_len[b] + k > c->p.max_seq) return fail(c, DEER_ECAPACITY, "sequence %d: length %d + k exceeds max_seq", b, c->h_len[b]);
        maxlim = std::max(maxlim, c->h_len[b] + k);
        any_ing |= c->h_ing_n[b] > 0;
    }
    Work &w = c->wk;
    double keys = 0;
    for (int b = 0; b < B; ++b) keys += c->h_len[b] + k;
    // pass s fixes block positions [lo, hi), lo = ceil(k (s-1) / n), hi = ceil(k s / n); the first pass also
    // ingests the committed tokens the drafter has not cached yet
    for (int s = 1; s <= n_passes; ++s) {
        const int lo = (k * (s - 1) + n_passes - 1) / n_passes, hi = (k * s + n_passes - 1) / n_passes;
        if (hi == lo) continue;
        const int tps = any_ing ? 2 : 1;
        PassRows pr{};
        pr.draft_pass = 1; pr.st = w.st; pr.tokens = draft_dev; pr.k = k; pr.nrows = 0; pr.vocab = c->p.drafter.vocab;
        pr.mask_id = c->p.mask_token_id; pr.tiles_per_seq = tps; pr.n_fixed = lo;
        LmPlan lm{true, 0, tps, B, k, T, seed, lo, T > 0.f};
        int rc = run_pass(c, DEER_DRAFTER, B * tps, maxlim, lm, keys, &pr);
        if (rc) return rc;
        hipLaunchKernelGGL(k_draft_finish, dim3(B), dim3(32), 0, c->stream, w.st, w.res[DEER_DRAFTER], draft_dev, k, lo);
        LAUNCHCHK(c, "k_draft_finish");
        any_ing = 0;   // the device-side counts were cleared by k_draft_finish
    }
    std::fill(c->h_ing_n.begin(), c->h_ing_n.end(), 0);
    c->cur_k = k;
    c->cur_T = T;
    c->state = ST_DRAFTED;
    return DEER_OK;
}

int deer_draft_block(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t *draft_dev) {
    return deer_draft_block_multipass(c, k, T, seed, 1, draft_dev);
}

int deer_verify_block(deer_ctx *c, int32_t k, float T, const int32_t *draft_dev) {
    if (!c) return DEER_EINVAL;
    if (!draft_dev || k < 1 || k > c->p.max_k || !(T >= 0.f)) return fail(c, DEER_EINVAL, "bad k, T or null pointer");
    if (c->state != ST_DRAFTED) return fail(c, DEER_ESTATE, "verify_block must follow draft_block");
    if (k != c->cur_k || T != c->cur_T) return fail(c, DEER_EINVAL, "k and T must match the draft_block call");
    const int B = c->batch;
    const int nrows = k + c->bonus;   // [x_j, y^_1 .. y^_{k-1}] and, with the bonus token, y^_k
    int maxlim = 0;
    for (int b = 0; b < B; ++b) maxlim = std::max(maxlim, c->h_len[b] - 1 + nrows);
    Work &w = c->wk;
    PassRows pr{};
    pr.draft_pass = 0; pr.st = w.st; pr.tokens = draft_dev; pr.k = k; pr.nrows = nrows; pr.vocab = c->p.target.vocab;
    pr.tiles_per_seq = 1;
    LmPlan lm{true, 0, 1, B, nrows, T, 0};
    double keys = 0;
    for (int b = 0; b < B; ++b) keys += c->h_len[b] - 1 + nrows;
    int rc = run_pass(c, DEER_TARGET, B, maxlim, lm, keys, &pr);
    if (rc) return rc;
    c->wk_draft = draft_dev;
    c->state = ST_VERIFIED;
    return DEER_OK;
}

// Shared by the two acceptance entry points: acc_part / acc_cnt are the sampling kernel's scratch (from the
// caller's workspace, or the library's static array).
static int accept_impl(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t *acc, int32_t *committed, int32_t *ncom,
                       AccPart *acc_part, int *acc_cnt, bool no_alloc) {
    if (!acc || !committed || !ncom || k < 1 || k > c->p.max_k || !(T >= 0.f)) return fail(c, DEER_EINVAL, "bad k, T or null pointer");
    if (c->state != ST_VERIFIED) return fail(c, DEER_ESTATE, "accept_and_commit must follow verify_block");
    if (k != c->cur_k || T != c->cur_T) return fail(c, DEER_EINVAL, "k and T must match the draft_block call");
    const int B = c->batch;
    Work &w = c->wk;
    const int V = c->p.target.vocab;
    const int cs = k + c->bonus;   // committed tokens per sequence: at most k, or k + 1 with the bonus token
    const char *d0 = (const char *)w.ao.accept_len;
    const size_t o_n = (const char *)w.ao.n_committed - d0, o_c = (const char *)w.ao.committed - d0;
    const size_t bytes = o_c + (size_t)B * cs * 4;
    char *host = c->h_pin;
    if (!host || bytes > c->h_pin_bytes) {
        if (no_alloc) return fail(c, DEER_ECAPACITY, "no page-locked result buffer was set up at init");
        c->h_ao.resize(bytes);
        host = c->h_ao.data();
    }
    if (T == 0.f)
        hipLaunchKernelGGL(k_accept_greedy, dim3(B), dim3(64), 0, c->stream, w.st, w.ao, c->wk_draft, w.res[DEER_TARGET], k,
                           c->p.eos_token_id, c->bonus);
    else
        hipLaunchKernelGGL(k_accept_sample, dim3(B, ACC_NB), dim3(1024), 0, c->stream, w.st, w.ao, c->wk_draft, w.res[DEER_TARGET],
                           w.res[DEER_DRAFTER], w.logits[DEER_TARGET], w.logits[DEER_DRAFTER], k, V, T, seed, c->p.eos_token_id,
                           c->bonus, acc_part, acc_cnt, w.rm.pos);
    LAUNCHCHK(c, "k_accept");
    // the three result arrays lie one after the other in the workspace: one copy instead of three
    HIPCHK(c, hipMemcpyAsync(host, d0, bytes, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    memcpy(acc, host, (size_t)B * 4);
    memcpy(ncom, host + o_n, (size_t)B * 4);
    memcpy(committed, host + o_c, (size_t)B * cs * 4);
    for (int b = 0; b < B; ++b) {
        c->h_len[b] += ncom[b];
        c->h_ing_n[b] = ncom[b];
        if (c->p.eos_token_id >= 0 && ncom[b] > 0 && committed[(size_t)b * cs + ncom[b] - 1] == c->p.eos_token_id) c->h_finished[b] = 1;
    }
    c->state = ST_PREFILLED;
    return DEER_OK;
}

int deer_accept_and_commit(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t *acc, int32_t *committed, int32_t *ncom) {
    if (!c) return DEER_EINVAL;
    return accept_impl(c, k, T, seed, acc, committed, ncom, c->wk.acc_part, c->wk.acc_cnt, false);
}

int deer_accept_and_commit_static(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t *acc, int32_t *committed, int32_t *ncom) {
    if (!c) return DEER_EINVAL;
    if (c->batch > STATIC_MAX_BATCH) return fail(c, DEER_ECAPACITY, "the static scratch holds %d sequences, the batch has %d", STATIC_MAX_BATCH, c->batch);
    if (!c->static_scratch) return fail(c, DEER_EHIP, "the static scratch was not resolved for device %d", c->p.device);
    AccPart *part = (AccPart *)c->static_scratch;
    int *cnt = (int *)((char *)c->static_scratch + STATIC_PART_BYTES);
    if (T > 0.f && c->state == ST_VERIFIED) {
        // the array keeps the last call's contents: the arrival counters of this batch start at zero (a fill kernel,
        // not a memset node); stale candidates are overwritten before the last arrival reads them
        hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(STATIC_MAX_BATCH), 0, c->stream, (uint32_t *)cnt, 0u, (size_t)c->batch);
        LAUNCHCHK(c, "k_fill_u32");
    }
    return accept_impl(c, k, T, seed, acc, committed, ncom, part, cnt, true);
}

int deer_set_bonus_token(deer_ctx *c, int enable) {
    if (!c) return DEER_EINVAL;
    if (c->state == ST_DRAFTED || c->state == ST_VERIFIED) return fail(c, DEER_ESTATE, "the bonus token cannot change inside an iteration");
    c->bonus = enable ? 1 : 0;
    return DEER_OK;
}

int deer_destroy(deer_ctx *c) {
    if (!c) return DEER_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    if (c->h_pin) (void)hipHostFree(c->h_pin);
    delete c;
    return DEER_OK;
}

const char *deer_last_error(const deer_ctx *c) { return c ? c->err.c_str() : g_init_error.c_str(); }

int deer_debug_get_logits(deer_ctx *c, int model, float *out, size_t n_floats) {
    if (!c) return DEER_EINVAL;
    if (!out || model < 0 || model > 1) return fail(c, DEER_EINVAL, "bad model or null pointer");
    if (c->cur_k < 1) return fail(c, DEER_ESTATE, "no pass has run yet");
    if (!c->p.keep_logits && c->cur_T == 0.f) return fail(c, DEER_ESTATE, "logits were not kept (keep_logits = 0 and T = 0)");
    const size_t n = (size_t)c->batch * (c->cur_k + (model == DEER_TARGET ? c->bonus : 0)) * c->p.target.vocab;
    if (n_floats < n) return fail(c, DEER_ECAPACITY, "output holds %zu floats, need %zu", n_floats, n);
    HIPCHK(c, hipMemcpyAsync(out, c->wk.logits[model], n * 4, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return DEER_OK;
}

int deer_debug_profile(deer_ctx *c, int enable) {
    if (!c) return DEER_EINVAL;
    prof_close(c);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->prof_on = enable != 0;
    c->prof.clear();
    c->ev_used = 0;
    return DEER_OK;
}

int deer_debug_profile_read(deer_ctx *c, int kernel_class, double *total_ms, int64_t *launches, double *bytes) {
    if (!c || !total_ms || !launches || !bytes) return DEER_EINVAL;
    prof_close(c);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    *total_ms = 0.0; *launches = 0; *bytes = 0.0;
    for (const auto &r : c->prof) {
        if (r.cls != kernel_class) continue;
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, r.a, r.b));
        *total_ms += ms; *launches += r.launches; *bytes += r.bytes;
    }
    return DEER_OK;
}

int deer_debug_gemm_stamps(deer_ctx *c, int model, int launch, uint64_t *stamps_host, int32_t max_blocks, int32_t *blocks) {
    if (!c) return DEER_EINVAL;
    if (model < 0 || model > 1) return fail(c, DEER_EINVAL, "bad model");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (blocks) *blocks = c->stamp_blocks;
    if (stamps_host && c->stamp_blocks > 0 && max_blocks > 0)
        HIPCHK(c, hipMemcpy(stamps_host, c->wk.stamps, (size_t)std::min(max_blocks, c->stamp_blocks) * 64, hipMemcpyDeviceToHost));
    c->stamp_model = model;
    c->stamp_launch = launch;
    c->stamp_blocks = 0;
    return DEER_OK;
}

int deer_debug_route_spread(deer_ctx *c, int enable) {
    if (!c) return DEER_EINVAL;
    c->route_spread = enable ? 1 : 0;
    return DEER_OK;
}

int deer_debug_experts_streamed(deer_ctx *c, int64_t *pairs) {
    if (!c || !pairs) return DEER_EINVAL;
    *pairs = 0;
    if (!c->wk.moe_touched) return DEER_OK;
    unsigned long long v = 0;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(&v, c->wk.moe_touched, 8, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemset(c->wk.moe_touched, 0, 8));
    *pairs = (int64_t)v;
    return DEER_OK;
}

int deer_debug_stream_read(deer_ctx *c, const void *buf_dev, size_t bytes, int32_t workgroups, int32_t nontemporal,
                           int32_t reps, float *ms_per_read) {
    if (!c || !ms_per_read) return DEER_EINVAL;
    if (!buf_dev || bytes < 16 || bytes % 16 || ((uintptr_t)buf_dev & 15)) return fail(c, DEER_EINVAL, "buffer must be 16-byte aligned, a multiple of 16 bytes");
    if (workgroups < 1 || workgroups > (1 << 20) || reps < 1 || reps > 10000) return fail(c, DEER_EINVAL, "bad workgroups / reps");
    if (c->prof_on) return fail(c, DEER_ESTATE, "launch timing is on");
    uint32_t *out = (uint32_t *)c->wk.stamps;   // a word of the debugging buffer
    const size_t n = bytes / 16;
    auto launch = [&]() {
        if (nontemporal) hipLaunchKernelGGL(k_stream_read<true>, dim3((unsigned)workgroups), dim3(512), 0, c->stream, (const u32x4 *)buf_dev, n, out);
        else hipLaunchKernelGGL(k_stream_read<false>, dim3((unsigned)workgroups), dim3(512), 0, c->stream, (const u32x4 *)buf_dev, n, out);
    };
    for (int i = 0; i < 3; ++i) launch();
    LAUNCHCHK(c, "k_stream_read");
    hipEvent_t e0 = prof_event(c), e1 = prof_event(c);
    if (!e0 || !e1) return fail(c, DEER_EHIP, "hipEventCreate failed");
    HIPCHK(c, hipEventRecord(e0, c->stream));
    for (int i = 0; i < reps; ++i) launch();
    HIPCHK(c, hipEventRecord(e1, c->stream));
    HIPCHK(c, hipEventSynchronize(e1));
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
    c->ev_used -= 2;   // the two events go back to the pool
    *ms_per_read = ms / (float)reps;
    return DEER_OK;
}

int deer_debug_gemm_tiled(deer_ctx *c, int min_tiles) {
    if (!c) return DEER_EINVAL;
    if (min_tiles < 0) return fail(c, DEER_EINVAL, "min_tiles must not be negative");
    c->tiled_min_tiles = min_tiles;
    return DEER_OK;
}

int deer_debug_force_commit(deer_ctx *c, const int32_t *tokens, const int32_t *n, int32_t stride) {
    if (!c) return DEER_EINVAL;
    if (!tokens || !n || stride < 1) return fail(c, DEER_EINVAL, "null pointer or bad stride");
    if (c->state != ST_VERIFIED) return fail(c, DEER_ESTATE, "force_commit stands in for accept_and_commit: it must follow verify_block");
    const int B = c->batch, cs = c->cur_k + c->bonus;
    if (stride > 32) return fail(c, DEER_EINVAL, "stride must be at most 32");
    for (int b = 0; b < B; ++b) {
        if (n[b] < 0 || n[b] > cs || n[b] > stride) return fail(c, DEER_EINVAL, "sequence %d: %d tokens, at most %d fit this block", b, n[b], std::min(cs, stride));
        for (int i = 0; i < n[b]; ++i)
            if (tokens[(size_t)b * stride + i] < 0 || tokens[(size_t)b * stride + i] >= c->p.target.vocab) return fail(c, DEER_EINVAL, "token id outside the vocabulary");
    }
    Work &w = c->wk;
    // staged through the acceptance result arrays (unused until the next accept_and_commit)
    HIPCHK(c, hipMemcpyAsync(w.ao.committed, tokens, (size_t)B * stride * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(w.ao.n_committed, n, (size_t)B * 4, hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(k_force_commit, dim3((B + 63) / 64), dim3(64), 0, c->stream, w.st, w.ao.committed, w.ao.n_committed, stride,
                       c->p.eos_token_id, B);
    LAUNCHCHK(c, "k_force_commit");
    HIPCHK(c, hipStreamSynchronize(c->stream));   // the host arrays may be reused by the caller
    for (int b = 0; b < B; ++b) {
        c->h_len[b] += n[b];
        c->h_ing_n[b] = n[b];
        for (int i = 0; i < n[b]; ++i)
            if (c->p.eos_token_id >= 0 && tokens[(size_t)b * stride + i] == c->p.eos_token_id) c->h_finished[b] = 1;
    }
    c->state = ST_PREFILLED;
    return DEER_OK;
}

int deer_debug_load_kv(deer_ctx *c, int model, int32_t layer, int32_t seq, int32_t first_slot, int32_t n_slots,
                       const void *k_rows_dev, const void *v_rows_dev) {
    if (!c) return DEER_EINVAL;
    if (model < 0 || model > 1 || !k_rows_dev || !v_rows_dev) return fail(c, DEER_EINVAL, "bad model or null pointer");
    ModelRT &m = c->m[model];
    if (layer < 0 || layer >= m.c.n_layers || seq < 0 || seq >= c->p.max_batch) return fail(c, DEER_EINVAL, "layer or sequence out of range");
    if (first_slot < 0 || n_slots < 0 || (int64_t)first_slot + n_slots > c->p.max_seq) return fail(c, DEER_ECAPACITY, "slots %d .. %d exceed max_seq %d", first_slot, first_slot + n_slots, c->p.max_seq);
    if (n_slots == 0) return DEER_OK;
    const KvView kv{m.kv + m.kv_k_base + (size_t)layer * m.kv_layer_stride, m.kv + m.kv_v_base + (size_t)layer * m.kv_layer_stride,
                    m.kv_seq_stride, m.kv_head_stride, c->p.max_seq};
    const size_t items = (size_t)n_slots * m.c.n_kv_heads * (m.c.head_dim / 8);
    hipLaunchKernelGGL(k_load_kv, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, c->stream, (const uint16_t *)k_rows_dev,
                       (const uint16_t *)v_rows_dev, kv, seq, first_slot, n_slots, m.c.n_kv_heads, m.c.head_dim);
    LAUNCHCHK(c, "k_load_kv");
    return DEER_OK;
}

int deer_get_lengths(const deer_ctx *c, int32_t *len) {
    if (!c || !len) return DEER_EINVAL;
    for (int b = 0; b < c->batch; ++b) len[b] = c->h_len[b];
    return DEER_OK;
}

int deer_get_kv_layout(const deer_ctx *c, int model, deer_kv_layout *out) {
    if (!c || !out || model < 0 || model > 1) return DEER_EINVAL;
    const ModelRT &m = c->m[model];
    out->k_base = m.kv_k_base; out->v_base = m.kv_v_base;
    out->layer_stride = m.kv_layer_stride; out->seq_stride = m.kv_seq_stride; out->head_stride = m.kv_head_stride;
    out->max_seq = c->p.max_seq; out->head_dim = m.c.head_dim;
    return DEER_OK;
}

}  // extern "C"
