// C ABI of the GELO library (see include/gelo.h): argument checks, the life cycle of
// contexts and per-batch mixing objects, and the kernel sequences behind each call.
// The call structure follows the three phases of the protocol (Section 3.2):
// trusted side (sample, mix) -> accelerator (project) -> trusted side (unmix).
#include "../../include/gelo.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <new>
#include <cstring>
#include <string>
#include <vector>

#include "gelo_internal.h"

using namespace gelo;

namespace {
constexpr float kConditionedBeta = 0.25f;
constexpr int kKappaSteps = 20;          // Lanczos steps of the condition estimate
constexpr uint32_t kStreamMixing = 0, kStreamShield = 1, kStreamPerturb = 2, kStreamBlock = 5;   // (3, 4: the structured kind)
// GAUSSIAN draws are accepted or rejected by their condition number, and a draw's chain of small
// launches leaves most of the chip idle: up to kLanes consecutive attempts are factorised side by
// side on library-owned streams, each in a workspace of its own, and the first acceptable one in
// attempt order wins - the same matrix a one-at-a-time loop would return.
constexpr int kLanes = 4;
constexpr int kQrSideBySide = 32;       // batched ORTHOGONAL draws: factorisations that share each launch, at most
constexpr size_t kQrSideBytes = (size_t)4 << 30;   // ... and no more of them than fit this much workspace
// how many factorisations of an n x n matrix a batched draw of `count` runs side by side
static int qr_side_by_side(int count, size_t ws_bytes) {
    int side = count < kQrSideBySide ? count : kQrSideBySide;
    const size_t fit = kQrSideBytes / ws_bytes;
    if ((size_t)side > fit) side = fit < 1 ? 1 : (int)fit;
    return side;
}
constexpr int kLanesMaxN = 1024;        // beyond this the rule is infeasible anyway and the buffers get large
// The condition estimate is a largest Ritz value, which approaches kappa_2 from below (measured within
// 0.5 % after kKappaSteps steps): a draw is accepted only if the estimate, raised by this margin, still
// meets the bound, so that an accepted A really satisfies kappa_2(A) <= cond_max.
constexpr float kKappaGuard = 1.01f;
// "Never reused" without a growing set: every id below `batch_floor` or more than kBatchWindow below the
// highest id seen counts as used; inside the window one bit per id remembers which ones were.
constexpr int kBatchWindow = 4096;

// Scratch of the entry point that allocates nothing (gelo_qkv_forward_static): the mixing matrices, the
// factorisation workspace and the shield buffers of one decode-shaped batch.  Host code never uses this
// name as an address: gelo_create asks the runtime for the array's device address, per device.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr int kStaticMaxDevices = 16;
}

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
void* g_scratch_ptr[kStaticMaxDevices] = {};
}

struct gelo_mixing {
    int kind, n_data, k, n, d, dtype;
    int64_t ldk;                 // leading dimension of A / A^-1 (n rounded up to 64), zero padded
    void* block;                 // one device allocation holding everything below
    size_t block_bytes;
    float* A32; float* Ainv32;   // dense kinds only
    uint16_t* A16; uint16_t* Ainv16;
    uint32_t* table;             // STRUCTURED only: its permutations and sign flips, nothing dense is kept
    bool structured;
    bool blocked;                // BLOCK_ORTHOGONAL: A32 ... Ainv16 hold the blocks one below the other, GELO_BLOCK_ROWS columns wide
    float* GS;                   // k x d shield directions
    float* gsnorm;               // k
    void* S;                     // k x d shield rows in the compute dtype
    float* rownorm;              // n_data
    float* stat;                 // [1] kappa estimate, [2..3] row-norm statistic of H as two halves (see norm_statistic)
    int attempt;
    float kappa;                 // host copy (GAUSSIAN); < 0: still only on the device
    bool in_use, mixed, consumed;
    uint64_t batch_id;
    hipEvent_t ready;            // recorded when sampling has been enqueued
    hipEvent_t released;         // recorded when the object went back to the pool
    hipStream_t sample_stream, last_stream;
};

struct gelo_ctx {
    int device;
    uint64_t seed;
    bool allow_reuse;
    uint64_t batch_floor;              // ids below it are refused (a resumed context starts here)
    uint64_t batch_high;               // one past the highest id used so far
    uint64_t batch_bits[kBatchWindow / 64];   // bit (id % kBatchWindow): id was used, for ids in [batch_high - kBatchWindow, batch_high)
    void* static_scratch;              // device address of `scratch` on this context's device
    std::string err;
    void* factor_ws; size_t factor_ws_bytes;
    void* chain_ws;  size_t chain_ws_bytes;
    void* quant_ws;  size_t quant_ws_bytes;    // FP8 projection: codes and row scales of the current U
    void* project_ws; size_t project_ws_bytes; // bf16 projection of at most 128 rows: float partial sums of the K slices
    float* host_scalars;         // pinned: kappa read-back, one slot per lane
    int* host_flag;
    std::vector<gelo_mixing*> pool;
    hipStream_t lane_stream[kLanes];   // created on the first GAUSSIAN draw
    hipEvent_t lane_fork, lane_done[kLanes];
    hipEvent_t lane_join;              // the winner's copies out of `cand` (on the caller's stream) are done
    bool lanes_ready, join_pending;
    void* cand; size_t cand_bytes;     // per lane: candidate A, A^-1 (float, and bf16 copies)
    // Everything of an attempt behind the Gaussian fill (about 125 launches that depend on nothing but
    // the lane's buffers) is captured once per lane into a graph and replayed: the host then spends one
    // launch instead of 125 per attempt, which is what lets four lanes really run side by side.
    hipGraphExec_t lane_graph[kLanes];
    bool lane_graph_ok[kLanes];
    int graph_n; bool graph_bf; void* graph_ws; void* graph_cand;   // what the graphs were captured for
    bool use_graphs;                   // off when GELO_EAGER_ATTEMPTS is set in the environment (tests compare the two)
};

namespace {

gelo_status fail(gelo_ctx* ctx, gelo_status st, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return st;
}

gelo_status hip_fail(gelo_ctx* ctx, hipError_t e, const char* what) {
    return fail(ctx, GELO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define GELO_HIP(ctx, expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_fail(ctx, e_, #expr); } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t elem_size(int dtype) { return dtype == GELO_BF16 ? 2 : 4; }
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

// Has batch id `b` been used on this context (or must it be assumed so)?  Pure: changes nothing.
bool batch_used(const gelo_ctx* ctx, uint64_t b) {
    if (ctx->allow_reuse) return false;
    if (b < ctx->batch_floor) return true;
    if (b >= ctx->batch_high) return false;
    if (ctx->batch_high - b > (uint64_t)kBatchWindow) return true;        // too far back to remember: assume used
    return (ctx->batch_bits[(b % kBatchWindow) / 64] >> (b % 64)) & 1u;
}

// Records `b` as used; ids the window slides over on the way up start out unused.
void batch_commit(gelo_ctx* ctx, uint64_t b) {
    if (ctx->allow_reuse) return;
    if (b >= ctx->batch_high) {
        if (b - ctx->batch_high >= (uint64_t)kBatchWindow) {
            std::memset(ctx->batch_bits, 0, sizeof ctx->batch_bits);
        } else {
            for (uint64_t i = ctx->batch_high; i <= b; ++i) ctx->batch_bits[(i % kBatchWindow) / 64] &= ~((uint64_t)1 << (i % 64));
        }
        ctx->batch_high = b + 1;
    }
    ctx->batch_bits[(b % kBatchWindow) / 64] |= (uint64_t)1 << (b % 64);
}

gelo_status grow(gelo_ctx* ctx, void** buf, size_t* have, size_t need) {
    if (*have >= need) return GELO_OK;
    if (*buf) {
        GELO_HIP(ctx, hipDeviceSynchronize());      // kernels of earlier calls may still use the old buffer
        GELO_HIP(ctx, hipFree(*buf));
        *buf = nullptr; *have = 0;
    }
    hipError_t e = hipMalloc(buf, need);
    if (e != hipSuccess) { *buf = nullptr; return fail(ctx, GELO_ENOMEM, "hipMalloc(%zu) failed: %s", need, hipGetErrorString(e)); }
    *have = need;
    return GELO_OK;
}

// Sizes of the device block behind one mixing object and where its parts sit in it.
struct MixingLayout { size_t mat32, mat16, tab, gs, s, gsnorm, rownorm, total; };

enum MixingForm { kDense = 0, kStructuredForm = 1, kBlocked = 2 };
inline MixingForm form_of(gelo_kind kind) {
    return kind == GELO_STRUCTURED ? kStructuredForm : kind == GELO_BLOCK_ORTHOGONAL ? kBlocked : kDense;
}

MixingLayout mixing_layout(int n_data, int k, int d, int dtype, MixingForm form) {
    MixingLayout L;
    const bool structured = form == kStructuredForm;
    const int n = n_data + k;
    const int64_t ldk = form == kBlocked ? GELO_BLOCK_ROWS : round_up(n, 64);
    L.mat32 = structured ? 0 : up256((size_t)n * ldk * 4);
    L.mat16 = (structured || dtype != GELO_BF16) ? 0 : up256((size_t)n * ldk * 2);
    L.tab = structured ? up256(structured_table_words(n, kStructuredRounds) * 4) : 0;
    L.gs = up256((size_t)(k > 0 ? k : 1) * d * 4);
    L.s = up256((size_t)(k > 0 ? k : 1) * d * elem_size(dtype));
    L.gsnorm = up256((size_t)(k + 1) * 4);
    L.rownorm = up256((size_t)n_data * 4);
    L.total = 2 * L.mat32 + 2 * L.mat16 + L.tab + L.gs + L.s + L.gsnorm + L.rownorm + 256;
    return L;
}

// Fills the shape fields of `m` and points its buffers into the device block at `base` (L.total bytes).
void carve_mixing(gelo_mixing* m, void* base, int n_data, int k, int d, int dtype, MixingForm form) {
    const MixingLayout L = mixing_layout(n_data, k, d, dtype, form);
    m->n_data = n_data; m->k = k; m->n = n_data + k; m->d = d; m->dtype = dtype;
    m->structured = form == kStructuredForm; m->blocked = form == kBlocked;
    m->ldk = form == kBlocked ? GELO_BLOCK_ROWS : round_up(m->n, 64);
    m->block = base; m->block_bytes = L.total;
    char* p = (char*)base;
    m->A32 = (float*)p; p += L.mat32;
    m->Ainv32 = (float*)p; p += L.mat32;
    m->A16 = m->Ainv16 = nullptr;
    if (L.mat16) { m->A16 = (uint16_t*)p; p += L.mat16; m->Ainv16 = (uint16_t*)p; p += L.mat16; }
    m->table = (uint32_t*)p; p += L.tab;
    m->GS = (float*)p; p += L.gs;
    m->S = p; p += L.s;
    m->gsnorm = (float*)p; p += L.gsnorm;
    m->rownorm = (float*)p; p += L.rownorm;
    m->stat = (float*)p;
}

// Where the buffers a batched small draw fills sit inside a mixing object's block (the same for every object of a shape).
void small_targets_layout(const gelo_mixing* m, SmallSampleTargets* t) {
    const char* base = (const char*)m->block;
    t->off_A32 = (const char*)m->A32 - base; t->off_Ainv32 = (const char*)m->Ainv32 - base;
    t->off_A16 = m->A16 ? (const char*)m->A16 - base : -1; t->off_Ainv16 = m->Ainv16 ? (const char*)m->Ainv16 - base : -1;
    t->off_GS = (const char*)m->GS - base; t->off_gsnorm = (const char*)m->gsnorm - base;
}

// A free pooled object of this shape, or a new one (the only place a mixing object allocates; gelo_reserve
// fills the pool ahead of time so that the per-batch calls find one).
gelo_status acquire_mixing(gelo_ctx* ctx, int n_data, int k, int d, int dtype, MixingForm form, gelo_mixing** out) {
    for (gelo_mixing* m : ctx->pool) {
        if (!m->in_use && m->n_data == n_data && m->k == k && m->d == d && m->dtype == dtype &&
            m->structured == (form == kStructuredForm) && m->blocked == (form == kBlocked)) { *out = m; return GELO_OK; }
    }
    gelo_mixing* m = new (std::nothrow) gelo_mixing();
    if (!m) return fail(ctx, GELO_ENOMEM, "host allocation failed");
    const MixingLayout L = mixing_layout(n_data, k, d, dtype, form);
    void* block = nullptr;
    hipError_t e = hipMalloc(&block, L.total);
    if (e != hipSuccess) { delete m; return fail(ctx, GELO_ENOMEM, "hipMalloc(%zu) failed: %s", L.total, hipGetErrorString(e)); }
    carve_mixing(m, block, n_data, k, d, dtype, form);
    if (hipEventCreateWithFlags(&m->ready, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->released, hipEventDisableTiming) != hipSuccess) {
        hipFree(m->block); delete m;
        return fail(ctx, GELO_EHIP, "hipEventCreate failed");
    }
    m->last_stream = nullptr;
    ctx->pool.push_back(m);
    *out = m;
    return GELO_OK;
}

void drop_lane_graphs(gelo_ctx* ctx) {
    for (int i = 0; i < kLanes; ++i) {
        if (ctx->lane_graph_ok[i]) (void)hipGraphExecDestroy(ctx->lane_graph[i]);
        ctx->lane_graph_ok[i] = false;
    }
}

gelo_status ensure_lanes(gelo_ctx* ctx) {
    if (ctx->lanes_ready) return GELO_OK;
    GELO_HIP(ctx, hipEventCreateWithFlags(&ctx->lane_fork, hipEventDisableTiming));
    GELO_HIP(ctx, hipEventCreateWithFlags(&ctx->lane_join, hipEventDisableTiming));
    for (int i = 0; i < kLanes; ++i) {
        GELO_HIP(ctx, hipStreamCreateWithFlags(&ctx->lane_stream[i], hipStreamNonBlocking));
        GELO_HIP(ctx, hipEventCreateWithFlags(&ctx->lane_done[i], hipEventDisableTiming));
    }
    ctx->lanes_ready = true;
    return GELO_OK;
}

bool owns(const gelo_ctx* ctx, const gelo_mixing* m) {
    for (const gelo_mixing* q : ctx->pool) if (q == m) return true;
    return false;
}

gelo_status run_gemm(gelo_ctx* ctx, int dtype, const GemmOperands& g, hipStream_t s) {
    hipError_t e = dtype == GELO_BF16 ? gemm_bf16(g, s) : gemm_f32(g, s);
    if (e != hipSuccess) return hip_fail(ctx, e, "GEMM launch");
    return GELO_OK;
}

// The products of a block-diagonal mix or unmix: bf16 in one launch, float one product at a time.
gelo_status run_gemm_blocks(gelo_ctx* ctx, int dtype, const GemmOperands* ops, int count, hipStream_t s) {
    if (count == 0) return GELO_OK;
    if (dtype == GELO_BF16) {
        const hipError_t e = gemm_bf16_batched(ops, count, s);
        if (e != hipSuccess) return hip_fail(ctx, e, "batched GEMM launch");
        return GELO_OK;
    }
    for (int i = 0; i < count; ++i) {
        const gelo_status st = run_gemm(ctx, dtype, ops[i], s);
        if (st != GELO_OK) return st;
    }
    return GELO_OK;
}

gelo_status check_matrix(gelo_ctx* ctx, const char* name, const void* p, int64_t ld, int cols) {
    if (!p) return fail(ctx, GELO_EINVAL, "%s is NULL", name);
    if (!aligned16(p)) return fail(ctx, GELO_EALIGN, "%s is not 16-byte aligned", name);
    if (ld < cols) return fail(ctx, GELO_EINVAL, "leading dimension of %s (%lld) is below its width (%d)", name, (long long)ld, cols);
    if (ld % 8 != 0) return fail(ctx, GELO_EALIGN, "leading dimension of %s (%lld) is not a multiple of 8", name, (long long)ld);
    return GELO_OK;
}

}  // namespace

extern "C" {

const char* gelo_status_string(gelo_status s) {
    switch (s) {
        case GELO_OK: return "ok";
        case GELO_EINVAL: return "invalid argument";
        case GELO_ESHAPE: return "unsupported shape";
        case GELO_EDTYPE: return "dtype mismatch";
        case GELO_EALIGN: return "misaligned pointer or leading dimension";
        case GELO_ENOMEM: return "out of memory";
        case GELO_ECOND: return "no well-conditioned draw within the attempt budget";
        case GELO_ESINGULAR: return "singular mixing matrix";
        case GELO_EREUSE: return "batch id or mixing object reused";
        case GELO_ESTATE: return "call out of order";
        case GELO_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

gelo_status gelo_create(gelo_ctx** out, int device, uint64_t seed, int allow_batch_reuse) {
    if (!out) return GELO_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return GELO_EINVAL;
    if (hipSetDevice(device) != hipSuccess) return GELO_EHIP;
    gelo_ctx* ctx = new (std::nothrow) gelo_ctx();
    if (!ctx) return GELO_ENOMEM;
    ctx->device = device; ctx->seed = seed; ctx->allow_reuse = allow_batch_reuse != 0;
    ctx->batch_floor = 0; ctx->batch_high = 0;
    std::memset(ctx->batch_bits, 0, sizeof ctx->batch_bits);
    // the device address of the static scratch array, asked for once per device with that device current
    ctx->static_scratch = device < kStaticMaxDevices ? g_scratch_ptr[device] : nullptr;
    if (!ctx->static_scratch) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { delete ctx; return GELO_EHIP; }
        ctx->static_scratch = ptr;
        if (device < kStaticMaxDevices) g_scratch_ptr[device] = ptr;
    }
    ctx->factor_ws = ctx->chain_ws = nullptr; ctx->factor_ws_bytes = ctx->chain_ws_bytes = 0;
    ctx->quant_ws = nullptr; ctx->quant_ws_bytes = 0;
    ctx->project_ws = nullptr; ctx->project_ws_bytes = 0;
    ctx->host_scalars = nullptr; ctx->host_flag = nullptr;
    ctx->lanes_ready = false; ctx->join_pending = false; ctx->cand = nullptr; ctx->cand_bytes = 0;
    for (int i = 0; i < kLanes; ++i) ctx->lane_graph_ok[i] = false;
    ctx->graph_n = 0; ctx->graph_bf = false; ctx->graph_ws = ctx->graph_cand = nullptr;
    ctx->use_graphs = std::getenv("GELO_EAGER_ATTEMPTS") == nullptr;
    if (hipHostMalloc((void**)&ctx->host_scalars, 64, hipHostMallocDefault) != hipSuccess) { delete ctx; return GELO_ENOMEM; }
    ctx->host_flag = (int*)(ctx->host_scalars + 8);
    if (gemm_bf16_init() != hipSuccess || gemm_f32_init() != hipSuccess || lu_init() != hipSuccess ||
        structured_init() != hipSuccess || small_init() != hipSuccess || gemm_fp8_init() != hipSuccess ||
        factor_init() != hipSuccess || sampler_init() != hipSuccess) {
        hipHostFree(ctx->host_scalars); delete ctx; return GELO_EHIP;
    }
    *out = ctx;
    return GELO_OK;
}

gelo_status gelo_destroy(gelo_ctx* ctx) {
    if (!ctx) return GELO_EINVAL;
    hipSetDevice(ctx->device);
    hipDeviceSynchronize();
    for (gelo_mixing* m : ctx->pool) {
        hipEventDestroy(m->ready); hipEventDestroy(m->released);
        hipFree(m->block);
        delete m;
    }
    drop_lane_graphs(ctx);
    if (ctx->lanes_ready) {
        (void)hipEventDestroy(ctx->lane_fork); (void)hipEventDestroy(ctx->lane_join);
        for (int i = 0; i < kLanes; ++i) { (void)hipStreamDestroy(ctx->lane_stream[i]); (void)hipEventDestroy(ctx->lane_done[i]); }
    }
    if (ctx->cand) (void)hipFree(ctx->cand);
    if (ctx->factor_ws) (void)hipFree(ctx->factor_ws);
    if (ctx->chain_ws) (void)hipFree(ctx->chain_ws);
    if (ctx->quant_ws) (void)hipFree(ctx->quant_ws);
    if (ctx->project_ws) (void)hipFree(ctx->project_ws);
    if (ctx->host_scalars) (void)hipHostFree(ctx->host_scalars);
    delete ctx;
    return GELO_OK;
}

const char* gelo_last_error(const gelo_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

// BLOCK_ORTHOGONAL: block i owns mixed rows [row0, row0 + rows), rows = min(GELO_BLOCK_ROWS, n - row0), mixes data rows
// [data0, data0 + data_rows) with shield rows [shield0, shield0 + shield_rows); of the rows up to a cut r,
// floor(k r / n) are shield rows.
struct BlockPiece { int row0, rows, data0, data_rows, shield0, shield_rows; };
static int block_count(int n) { return (n + GELO_BLOCK_ROWS - 1) / GELO_BLOCK_ROWS; }
static_assert((GELO_MAX_N + GELO_BLOCK_ROWS - 1) / GELO_BLOCK_ROWS <= kGemmBatchMax, "one batched launch takes all blocks");
static BlockPiece block_piece(int n_data, int k, int i) {
    const int n = n_data + k;
    const int r0 = i * GELO_BLOCK_ROWS, r1 = r0 + GELO_BLOCK_ROWS < n ? r0 + GELO_BLOCK_ROWS : n;
    const int s0 = (int)((int64_t)k * r0 / n), s1 = (int)((int64_t)k * r1 / n);
    BlockPiece b;
    b.row0 = r0; b.rows = r1 - r0; b.shield0 = s0; b.shield_rows = s1 - s0;
    b.data0 = r0 - s0; b.data_rows = b.rows - b.shield_rows;
    return b;
}
// factorisation workspaces of all blocks, one behind the other: the full blocks first (they share their launches)
static size_t block_workspace_bytes(int n) {
    const int full = n / GELO_BLOCK_ROWS, rest = n % GELO_BLOCK_ROWS;
    return (size_t)full * up256(factor_workspace_bytes(GELO_BLOCK_ROWS)) + (rest ? up256(factor_workspace_bytes(rest)) : 0);
}

// Argument checks shared by the sampling entry points; on success *n_out = n_data + k_shield.
static gelo_status check_sample_args(gelo_ctx* ctx, gelo_kind kind, int n_data, int k_shield, int d, gelo_dtype dtype,
                                     double cond_max, int max_attempts, uint64_t batch_id, int* n_out) {
    if (kind != GELO_ORTHOGONAL && kind != GELO_GAUSSIAN && kind != GELO_CONDITIONED && kind != GELO_STRUCTURED &&
        kind != GELO_BLOCK_ORTHOGONAL && kind != GELO_REFLECTOR_PRODUCT)
        return fail(ctx, GELO_EINVAL, "unknown kind %d", (int)kind);
    if (dtype != GELO_F32 && dtype != GELO_BF16) return fail(ctx, GELO_EINVAL, "unknown dtype %d", (int)dtype);
    if (n_data < 1 || k_shield < 0 || d < 1) return fail(ctx, GELO_EINVAL, "n_data=%d k_shield=%d d=%d", n_data, k_shield, d);
    if (d % 8 != 0) return fail(ctx, GELO_EALIGN, "d=%d is not a multiple of 8", d);
    const int64_t n64 = (int64_t)n_data + k_shield;
    if (n64 > GELO_MAX_N) return fail(ctx, GELO_ESHAPE, "n = n_data + k_shield = %lld exceeds GELO_MAX_N = %d", (long long)n64, GELO_MAX_N);
    const int n = (int)n64;
    if (kind == GELO_STRUCTURED && n > structured_max_rows())
        return fail(ctx, GELO_ESHAPE, "n = %d exceeds what one workgroup's LDS holds for the structured kind (%d)", n, structured_max_rows());
    if (kind == GELO_GAUSSIAN) {
        if (!(cond_max >= 1.0)) return fail(ctx, GELO_EINVAL, "cond_max=%g must be >= 1", cond_max);
        if (max_attempts < 1 || max_attempts > GELO_MAX_ATTEMPTS) return fail(ctx, GELO_EINVAL, "max_attempts=%d outside 1..%d", max_attempts, GELO_MAX_ATTEMPTS);
    }
    if (batch_id == UINT64_MAX) return fail(ctx, GELO_EINVAL, "batch id 2^64 - 1 is reserved");
    if (batch_used(ctx, batch_id))
        return fail(ctx, GELO_EREUSE, "batch id %llu was already used on this context (or lies below its floor / window)", (unsigned long long)batch_id);
    *n_out = n;
    return GELO_OK;
}

// Enqueues the draw of batch `batch_id` into the buffers `m` points at, with `ws` as factorisation
// workspace (not used by STRUCTURED).  `lanes` > 1 (GAUSSIAN only) uses the context's lane buffers, which
// the caller has sized.  Allocates nothing.
static gelo_status sample_into(gelo_ctx* ctx, gelo_mixing* m, FactorWorkspace ws, size_t ws_bytes, int lanes, gelo_kind kind,
                               double cond_max, int max_attempts, uint64_t batch_id, hipStream_t s) {
    const int n = m->n, k_shield = m->k, d = m->d;
    const bool structured = kind == GELO_STRUCTURED;
    gelo_status st = GELO_OK;
    PhiloxStream ps;
    ps.key0 = (uint32_t)ctx->seed; ps.key1 = (uint32_t)(ctx->seed >> 32);
    ps.c2 = (uint32_t)batch_id; ps.c3 = (uint32_t)(batch_id >> 32);
    const int64_t ld = ws.ld, ldk = m->ldk;
    const bool bf = m->dtype == GELO_BF16;
    m->kind = kind; m->attempt = 0; m->kappa = 1.0f;

    auto orthogonal_into_X = [&](bool direct) -> hipError_t {
        ps.c1 = kStreamMixing << 8;
        // straight into the QR's tiles; the product of reflectors reads column k from row k down only
        hipError_t e = fill_normal(ws.M, ws.n_pad / 16, n, n, ps, 1.0f, direct ? 2 : 1, s);
        if (e == hipSuccess) e = householder_qr(ws, n, 1, 0, s, direct);
        return e;
    };

    if (kind == GELO_ORTHOGONAL && n <= kSmallMaxN) {
        // decode-shaped: Gaussian, QR, both matrices and the shield directions from one launch
        SmallSampleTargets t;
        small_targets_layout(m, &t);
        t.block[0] = m->block;
        ps.c1 = kStreamMixing << 8;
        GELO_HIP(ctx, small_sample(t, 1, batch_id, ps, kStreamShield << 8, n, k_shield, d, ldk, s));
        m->batch_id = batch_id;
        return GELO_OK;
    }
    if (structured) {
        GELO_HIP(ctx, structured_tables(m->table, n, kStructuredRounds, ps, s));
    } else if (kind == GELO_BLOCK_ORTHOGONAL) {
        // ws.M is the start of the blocks' workspaces here (block_workspace_bytes): the full blocks, whose
        // factorisations share their launches, then the last, shorter one
        constexpr int B = GELO_BLOCK_ROWS;
        char* base = (char*)ws.M;
        const int full = n / B, rest = n % B;
        const size_t wb = up256(factor_workspace_bytes(B));
        auto emit_block = [&](const FactorWorkspace& w, int i, int rows) {
            const int64_t at = (int64_t)i * B * ldk;
            return emit_matrix(w.X, w.n_pad / 16, 1, w.rdiag, rows, ldk, m->A32 + at, m->A16 ? m->A16 + at : nullptr,
                               m->Ainv32 + at, m->Ainv16 ? m->Ainv16 + at : nullptr, s);
        };
        FactorWorkspace w;
        for (int i = 0; i < full; ++i) {
            factor_workspace_carve(base + wb * i, B, &w);
            ps.c1 = (kStreamBlock << 8) | (uint32_t)i;
            GELO_HIP(ctx, fill_normal(w.M, w.n_pad / 16, B, B, ps, 1.0f, 1, s));
        }
        if (full > 0) {
            factor_workspace_carve(base, B, &w);
            GELO_HIP(ctx, householder_qr(w, B, full, (int64_t)(wb / sizeof(float)), s));
        }
        for (int i = 0; i < full; ++i) {
            factor_workspace_carve(base + wb * i, B, &w);
            GELO_HIP(ctx, emit_block(w, i, B));
        }
        if (rest > 0) {
            factor_workspace_carve(base + wb * full, rest, &w);
            ps.c1 = (kStreamBlock << 8) | (uint32_t)full;
            GELO_HIP(ctx, fill_normal(w.M, w.n_pad / 16, rest, rest, ps, 1.0f, 1, s));
            GELO_HIP(ctx, householder_qr(w, rest, 1, 0, s));
            GELO_HIP(ctx, emit_block(w, full, rest));
        }
    } else if (kind == GELO_ORTHOGONAL || kind == GELO_REFLECTOR_PRODUCT) {
        GELO_HIP(ctx, orthogonal_into_X(kind == GELO_REFLECTOR_PRODUCT));
        // A = Q diag(sign r_ii) (sign beta_k for the product of reflectors); A^-1 = A^T
        GELO_HIP(ctx, emit_matrix(ws.X, ws.n_pad / 16, 1, ws.rdiag, n, ldk, m->A32, m->A16, m->Ainv32, m->Ainv16, s));
    } else if (kind == GELO_CONDITIONED) {
        GELO_HIP(ctx, orthogonal_into_X(false));
        GELO_HIP(ctx, emit_matrix(ws.X, ws.n_pad / 16, 1, ws.rdiag, n, ldk, m->A32, nullptr, nullptr, nullptr, s));
        ps.c1 = kStreamPerturb << 8;
        GELO_HIP(ctx, fill_normal(ws.M, ld, n, n, ps, 1.0f, 0, s));
        GELO_HIP(ctx, axpy_matrix(m->A32, ldk, ws.M, ld, n, n, kConditionedBeta / std::sqrt((float)n), s));
        GELO_HIP(ctx, emit_matrix(m->A32, ldk, 0, nullptr, n, ld, ws.M, nullptr, nullptr, nullptr, s));
        if (bf) GELO_HIP(ctx, emit_matrix(m->A32, ldk, 0, nullptr, n, ldk, nullptr, m->A16, nullptr, nullptr, s));
        GELO_HIP(ctx, pad_matrix(ws.M, ld, n, ws.n_pad, 1, s));
        GELO_HIP(ctx, lu_inverse(ws, s));
        GELO_HIP(ctx, emit_matrix(ws.X, ld, 0, nullptr, n, ldk, m->Ainv32, m->Ainv16, nullptr, nullptr, s));
        GELO_HIP(ctx, kappa_estimate(m->A32, m->Ainv32, ldk, n, ws, kKappaSteps, s));
        GELO_HIP(ctx, hipMemcpyAsync(m->stat + 1, ws.scalars, sizeof(float), hipMemcpyDeviceToDevice, s));
        m->kappa = -1.0f;                                     // stays on the device until someone asks
    } else {
        // GAUSSIAN: groups of `lanes` consecutive attempts side by side; the host reads every lane's
        // kappa and singular flag (the library's only host synchronisation) and takes the first
        // acceptable attempt in order.
        const size_t mat32 = up256((size_t)n * ldk * 4), mat16 = bf ? up256((size_t)n * ldk * 2) : 0;
        const size_t lane_cand = 2 * mat32 + 2 * mat16;
        if (lanes > 1) {
            if (ctx->cand_bytes < lane_cand * lanes || !ctx->lanes_ready) return fail(ctx, GELO_ESTATE, "lane buffers were not prepared");
            if (ctx->graph_n != n || ctx->graph_bf != bf || ctx->graph_ws != ctx->factor_ws || ctx->graph_cand != ctx->cand) {
                drop_lane_graphs(ctx);      // captured for other buffers or another size
                ctx->graph_n = n; ctx->graph_bf = bf; ctx->graph_ws = ctx->factor_ws; ctx->graph_cand = ctx->cand;
            }
        }
        bool accepted = false, singular_last = false;
        for (int base = 0; base < max_attempts && !accepted; base += lanes) {
            const int count = max_attempts - base < lanes ? max_attempts - base : lanes;
            if (lanes > 1) GELO_HIP(ctx, hipEventRecord(ctx->lane_fork, s));
            FactorWorkspace lw[kLanes];
            float* cA32[kLanes]; float* cAi32[kLanes]; uint16_t* cA16[kLanes]; uint16_t* cAi16[kLanes];
            for (int i = 0; i < count; ++i) {
                hipStream_t ls = lanes > 1 ? ctx->lane_stream[i] : s;
                if (lanes > 1) {
                    GELO_HIP(ctx, hipStreamWaitEvent(ls, ctx->lane_fork, 0));
                    if (ctx->join_pending) GELO_HIP(ctx, hipStreamWaitEvent(ls, ctx->lane_join, 0));   // an earlier call may still be copying
                    factor_workspace_carve((char*)ctx->factor_ws + ws_bytes * i, n, &lw[i]);
                    char* c = (char*)ctx->cand + lane_cand * i;
                    cA32[i] = (float*)c; cAi32[i] = (float*)(c + mat32);
                    cA16[i] = bf ? (uint16_t*)(c + 2 * mat32) : nullptr;
                    cAi16[i] = bf ? (uint16_t*)(c + 2 * mat32 + mat16) : nullptr;
                } else {
                    lw[i] = ws; cA32[i] = m->A32; cAi32[i] = m->Ainv32; cA16[i] = m->A16; cAi16[i] = m->Ainv16;
                }
                ps.c1 = (kStreamMixing << 8) | (uint32_t)(base + i);
                GELO_HIP(ctx, fill_normal(lw[i].M, ld, n, n, ps, 1.0f / std::sqrt((float)n), 0, ls));
                // everything behind the fill: the same launches for every attempt of this lane
                auto factorise = [&]() -> hipError_t {
                    hipError_t e = emit_matrix(lw[i].M, ld, 0, nullptr, n, ldk, cA32[i], cA16[i], nullptr, nullptr, ls);
                    if (e == hipSuccess) e = pad_matrix(lw[i].M, ld, n, lw[i].n_pad, 1, ls);
                    if (e == hipSuccess) e = lu_inverse(lw[i], ls);
                    if (e == hipSuccess) e = emit_matrix(lw[i].X, ld, 0, nullptr, n, ldk, cAi32[i], cAi16[i], nullptr, nullptr, ls);
                    if (e == hipSuccess) e = kappa_estimate(cA32[i], cAi32[i], ldk, n, lw[i], kKappaSteps, ls);
                    if (e == hipSuccess) e = hipMemcpyAsync(ctx->host_scalars + i, lw[i].scalars, sizeof(float), hipMemcpyDeviceToHost, ls);
                    if (e == hipSuccess) e = hipMemcpyAsync(ctx->host_flag + i, lw[i].flag, sizeof(int), hipMemcpyDeviceToHost, ls);
                    return e;
                };
                if (lanes > 1 && ctx->use_graphs && !ctx->lane_graph_ok[i]) {
                    // a capture records and runs nothing; if the runtime refuses any part of it, this
                    // context goes back to launching every attempt kernel by kernel
                    hipGraph_t graph = nullptr;
                    bool ok = hipStreamBeginCapture(ls, hipStreamCaptureModeRelaxed) == hipSuccess;
                    if (ok) {
                        const hipError_t e_body = factorise();
                        const hipError_t e_end = hipStreamEndCapture(ls, &graph);      // also ends a failed capture
                        ok = e_body == hipSuccess && e_end == hipSuccess && graph != nullptr;
                    }
                    if (ok) ok = hipGraphInstantiate(&ctx->lane_graph[i], graph, nullptr, nullptr, 0) == hipSuccess;
                    if (graph) (void)hipGraphDestroy(graph);
                    if (ok) {
                        ctx->lane_graph_ok[i] = true;
                    } else {
                        (void)hipGetLastError();
                        ctx->use_graphs = false;
                    }
                }
                if (lanes > 1 && ctx->use_graphs && ctx->lane_graph_ok[i]) {
                    GELO_HIP(ctx, hipGraphLaunch(ctx->lane_graph[i], ls));
                } else {
                    GELO_HIP(ctx, factorise());
                }
                if (lanes > 1) GELO_HIP(ctx, hipEventRecord(ctx->lane_done[i], ls));
            }
            if (lanes > 1) {
                for (int i = 0; i < count; ++i) GELO_HIP(ctx, hipEventSynchronize(ctx->lane_done[i]));
            } else {
                GELO_HIP(ctx, hipStreamSynchronize(s));
            }
            for (int i = 0; i < count && !accepted; ++i) {
                singular_last = ctx->host_flag[i] != 0;
                const float kappa = ctx->host_scalars[i];
                if (singular_last || !(kappa * kKappaGuard <= (float)cond_max)) continue;
                accepted = true; m->attempt = base + i; m->kappa = kappa;
                GELO_HIP(ctx, hipMemcpyAsync(m->stat + 1, lw[i].scalars, sizeof(float), hipMemcpyDeviceToDevice, s));
                if (lanes > 1) {      // every lane has finished: plain copies on the caller's stream
                    GELO_HIP(ctx, hipMemcpyAsync(m->A32, cA32[i], (size_t)n * ldk * 4, hipMemcpyDeviceToDevice, s));
                    GELO_HIP(ctx, hipMemcpyAsync(m->Ainv32, cAi32[i], (size_t)n * ldk * 4, hipMemcpyDeviceToDevice, s));
                    if (bf) {
                        GELO_HIP(ctx, hipMemcpyAsync(m->A16, cA16[i], (size_t)n * ldk * 2, hipMemcpyDeviceToDevice, s));
                        GELO_HIP(ctx, hipMemcpyAsync(m->Ainv16, cAi16[i], (size_t)n * ldk * 2, hipMemcpyDeviceToDevice, s));
                    }
                    GELO_HIP(ctx, hipEventRecord(ctx->lane_join, s));
                    ctx->join_pending = true;
                }
            }
        }
        if (!accepted) {
            if (singular_last) return fail(ctx, GELO_ESINGULAR, "zero pivot in the last of %d draws", max_attempts);
            return fail(ctx, GELO_ECOND, "no draw with kappa <= %g within %d attempts", cond_max, max_attempts);
        }
    }
    if (k_shield > 0) {
        ps.c1 = kStreamShield << 8;
        GELO_HIP(ctx, shield_directions(m->GS, k_shield, d, ps, m->gsnorm, s));
    }
    (void)st; (void)structured;
    m->batch_id = batch_id;
    return GELO_OK;
}

// Device memory a draw of this shape needs beyond the mixing object: the factorisation workspace (one per
// lane) and, for side-by-side GAUSSIAN attempts, the candidate buffers and streams.
static gelo_status prepare_sampling(gelo_ctx* ctx, gelo_kind kind, int n, gelo_dtype dtype, int max_attempts, int* lanes_out) {
    const int lanes = (kind == GELO_GAUSSIAN && n <= kLanesMaxN) ? (max_attempts < kLanes ? max_attempts : kLanes) : 1;
    *lanes_out = lanes;
    if (kind == GELO_STRUCTURED) return GELO_OK;
    if (kind == GELO_BLOCK_ORTHOGONAL) return grow(ctx, &ctx->factor_ws, &ctx->factor_ws_bytes, block_workspace_bytes(n));
    gelo_status st = grow(ctx, &ctx->factor_ws, &ctx->factor_ws_bytes, up256(factor_workspace_bytes(n)) * lanes);
    if (st != GELO_OK || lanes == 1) return st;
    const int64_t ldk = round_up(n, 64);
    const size_t mat32 = up256((size_t)n * ldk * 4), mat16 = dtype == GELO_BF16 ? up256((size_t)n * ldk * 2) : 0;
    st = grow(ctx, &ctx->cand, &ctx->cand_bytes, (2 * mat32 + 2 * mat16) * lanes);
    if (st == GELO_OK) st = ensure_lanes(ctx);
    return st;
}

gelo_status gelo_sample_mixing(gelo_ctx* ctx, gelo_kind kind, int n_data, int k_shield, int d,
                               gelo_dtype dtype, double cond_max, int max_attempts,
                               uint64_t batch_id, gelo_mixing** out, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!out) return fail(ctx, GELO_EINVAL, "out is NULL");
    *out = nullptr;
    int n = 0;
    gelo_status st = check_sample_args(ctx, kind, n_data, k_shield, d, dtype, cond_max, max_attempts, batch_id, &n);
    if (st != GELO_OK) return st;
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    int lanes = 1;
    st = prepare_sampling(ctx, kind, n, dtype, max_attempts, &lanes);     // allocates on first use of a shape only (see gelo_reserve)
    if (st != GELO_OK) return st;
    FactorWorkspace ws = {};
    const size_t ws_bytes = up256(factor_workspace_bytes(n));
    if (kind == GELO_BLOCK_ORTHOGONAL) ws.M = (float*)ctx->factor_ws;      // sample_into carves the blocks' workspaces from here
    else if (kind != GELO_STRUCTURED) factor_workspace_carve(ctx->factor_ws, n, &ws);
    gelo_mixing* m = nullptr;
    st = acquire_mixing(ctx, n_data, k_shield, d, dtype, form_of(kind), &m);
    if (st != GELO_OK) return st;
    if (m->last_stream != nullptr || m->mixed) GELO_HIP(ctx, hipStreamWaitEvent(s, m->released, 0));
    st = sample_into(ctx, m, ws, ws_bytes, lanes, kind, cond_max, max_attempts, batch_id, s);
    if (st != GELO_OK) return st;
    GELO_HIP(ctx, hipEventRecord(m->ready, s));
    m->in_use = true; m->mixed = false; m->consumed = false;
    m->sample_stream = s; m->last_stream = s;
    batch_commit(ctx, batch_id);
    *out = m;
    return GELO_OK;
}

// Launches of eq. 1 / eqs. 7-8 on the buffers of `m`: shield rows, then U = A [H ; S].
static gelo_status mix_launch(gelo_ctx* ctx, gelo_mixing* m, const void* H, int64_t ldh, float shield_scale,
                              gelo_norm_stat stat, void* U, int64_t ldu, hipStream_t s) {
    const bool bf = m->dtype == GELO_BF16;
    if (bf && !m->structured && !m->blocked && m->n <= kSmallMaxN) {
        // decode-shaped: row norms, then statistic + shield rows + product in one launch
        if (m->k > 0) GELO_HIP(ctx, row_norms(H, 1, ldh, m->n_data, m->d, m->rownorm, s));
        GELO_HIP(ctx, small_mix(m->A16, m->ldk, (const uint16_t*)H, ldh, m->GS, m->gsnorm, m->rownorm, (int)stat, shield_scale,
                                m->n_data, m->k, m->d, (uint16_t*)m->S, (uint16_t*)U, ldu, s));
        return GELO_OK;
    }
    if (m->k > 0) {
        GELO_HIP(ctx, row_norms(H, bf, ldh, m->n_data, m->d, m->rownorm, s));
        GELO_HIP(ctx, norm_statistic(m->rownorm, m->n_data, (int)stat, m->stat + 2, s));
        GELO_HIP(ctx, make_shields(m->GS, m->d, m->gsnorm, m->stat + 2, shield_scale, m->k, m->d, m->S, bf, m->d, s));
    }
    if (m->structured) {
        StructuredOperands o;
        o.in0 = H; o.ld0 = ldh; o.rows0 = m->n_data;
        o.in1 = m->S; o.ld1 = m->d;
        o.out = U; o.ldo = ldu; o.rows_out = m->n;
        o.table = m->table; o.n = m->n; o.ncols = m->d; o.rounds = kStructuredRounds; o.transposed = false;
        GELO_HIP(ctx, structured_apply(o, bf, s));
        return GELO_OK;
    }
    if (m->blocked) {
        // block i: rows [row0, row0 + rows) of U = A_i [its data rows of H; its shield rows]
        const size_t es = elem_size(m->dtype);
        GemmOperands ops[kGemmBatchMax];
        const int nb = block_count(m->n);
        for (int i = 0; i < nb; ++i) {
            const BlockPiece b = block_piece(m->n_data, m->k, i);
            GemmOperands& g = ops[i];
            g.A = bf ? (const void*)(m->A16 + (int64_t)b.row0 * m->ldk) : (const void*)(m->A32 + (int64_t)b.row0 * m->ldk); g.lda = m->ldk;
            g.B0 = (const char*)H + (int64_t)b.data0 * ldh * es; g.ldb0 = ldh; g.K0 = b.data_rows;
            g.B1 = b.shield_rows > 0 ? (const void*)((const char*)m->S + (int64_t)b.shield0 * m->d * es) : g.B0; g.ldb1 = b.shield_rows > 0 ? m->d : ldh;
            g.C = (char*)U + (int64_t)b.row0 * ldu * es; g.ldc = ldu;
            g.M = b.rows; g.N = m->d; g.K = b.rows; g.a_zero_padded = true;
        }
        return run_gemm_blocks(ctx, m->dtype, ops, nb, s);
    }
    GemmOperands g;
    g.A = bf ? (const void*)m->A16 : (const void*)m->A32; g.lda = m->ldk;
    g.B0 = H; g.ldb0 = ldh; g.K0 = m->n_data;
    g.B1 = m->S; g.ldb1 = m->d;
    g.C = U; g.ldc = ldu;
    g.M = m->n; g.N = m->d; g.K = m->n; g.a_zero_padded = true;
    return run_gemm(ctx, m->dtype, g, s);
}

// Launches of eq. 3 with the shield rows dropped: Z = (A^-1 Y)[0:n_data, :].
static gelo_status unmix_launch(gelo_ctx* ctx, gelo_mixing* m, int p, const void* Y, int64_t ldy, void* Z, int64_t ldz,
                                hipStream_t s) {
    const bool bf = m->dtype == GELO_BF16;
    if (m->structured) {
        StructuredOperands o;
        o.in0 = Y; o.ld0 = ldy; o.rows0 = m->n;
        o.in1 = nullptr; o.ld1 = 0;
        o.out = Z; o.ldo = ldz; o.rows_out = m->n_data;      // the shield rows of A^T Y are never stored
        o.table = m->table; o.n = m->n; o.ncols = p; o.rounds = kStructuredRounds; o.transposed = true;
        GELO_HIP(ctx, structured_apply(o, bf, s));
        return GELO_OK;
    }
    if (m->blocked) {
        // block i: its data rows of Z = (the first data_rows rows of A_i^T) x rows [row0, row0 + rows) of Y
        const size_t es = elem_size(m->dtype);
        GemmOperands ops[kGemmBatchMax];
        int nb = 0;
        for (int i = 0; i < block_count(m->n); ++i) {
            const BlockPiece b = block_piece(m->n_data, m->k, i);
            if (b.data_rows == 0) continue;
            GemmOperands& g = ops[nb++];
            g.A = bf ? (const void*)(m->Ainv16 + (int64_t)b.row0 * m->ldk) : (const void*)(m->Ainv32 + (int64_t)b.row0 * m->ldk); g.lda = m->ldk;
            g.B0 = (const char*)Y + (int64_t)b.row0 * ldy * es; g.ldb0 = ldy; g.K0 = b.rows;
            g.B1 = g.B0; g.ldb1 = ldy;
            g.C = (char*)Z + (int64_t)b.data0 * ldz * es; g.ldc = ldz;
            g.M = b.data_rows; g.N = p; g.K = b.rows; g.a_zero_padded = true;
        }
        return run_gemm_blocks(ctx, m->dtype, ops, nb, s);
    }
    GemmOperands g;
    g.A = bf ? (const void*)m->Ainv16 : (const void*)m->Ainv32; g.lda = m->ldk;   // rows 0..n_data-1 of A^-1
    g.B0 = Y; g.ldb0 = ldy; g.K0 = m->n;
    g.B1 = Y; g.ldb1 = ldy;
    g.C = Z; g.ldc = ldz;
    g.M = m->n_data; g.N = p; g.K = m->n; g.a_zero_padded = true;
    return run_gemm(ctx, m->dtype, g, s);
}

gelo_status gelo_mix(gelo_ctx* ctx, gelo_mixing* m, gelo_dtype dtype, const void* H, int64_t ldh,
                     float shield_scale, gelo_norm_stat stat, void* U, int64_t ldu, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or freed");
    if (dtype != GELO_F32 && dtype != GELO_BF16) return fail(ctx, GELO_EINVAL, "unknown dtype %d", (int)dtype);
    if ((int)dtype != m->dtype) return fail(ctx, GELO_EDTYPE, "H and U are %s but the mixing object was drawn for %s", dtype == GELO_BF16 ? "bf16" : "f32", m->dtype == GELO_BF16 ? "bf16" : "f32");
    if (stat != GELO_NORM_MEDIAN && stat != GELO_NORM_MEAN) return fail(ctx, GELO_EINVAL, "unknown norm statistic %d", (int)stat);
    if (m->k > 0 && !(shield_scale > 0.f)) return fail(ctx, GELO_EINVAL, "shield_scale=%g must be positive", (double)shield_scale);
    gelo_status st = check_matrix(ctx, "H", H, ldh, m->d);
    if (st == GELO_OK) st = check_matrix(ctx, "U", U, ldu, m->d);
    if (st != GELO_OK) return st;
    if (!ctx->allow_reuse && m->mixed) return fail(ctx, GELO_EREUSE, "this mixing object has already mixed a batch");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    if (s != m->sample_stream) GELO_HIP(ctx, hipStreamWaitEvent(s, m->ready, 0));
    st = mix_launch(ctx, m, H, ldh, shield_scale, stat, U, ldu, s);
    if (st != GELO_OK) return st;
    m->mixed = true; m->last_stream = s;
    return GELO_OK;
}

// Eq. 2 with a caller-chosen workspace for the partial sums of a decode-shaped product (NULL: none, the product then
// runs without cutting K); allocates nothing.
static gelo_status project_launch(gelo_ctx* ctx, gelo_dtype dtype, int n, int d, int p, const void* U, int64_t ldu,
                                  const void* W, int64_t ldw, void* Y, int64_t ldy, void* ws, size_t ws_bytes, hipStream_t s) {
    GemmOperands g;
    g.A = U; g.lda = ldu;
    g.B0 = W; g.ldb0 = ldw; g.K0 = d;
    g.B1 = W; g.ldb1 = ldw;
    g.C = Y; g.ldc = ldy;
    g.M = n; g.N = p; g.K = d;
    g.splitk_ws = ws; g.splitk_ws_bytes = ws_bytes;
    return run_gemm(ctx, dtype, g, s);
}

static size_t project_ws_need(gelo_dtype dtype, int n, int d, int p) {
    return dtype == GELO_BF16 ? gemm_bf16_skinny_ws_bytes(n, p, d) : 0;
}

gelo_status gelo_project(gelo_ctx* ctx, gelo_dtype dtype, int n, int d, int p,
                         const void* U, int64_t ldu, const void* W, int64_t ldw,
                         void* Y, int64_t ldy, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (dtype != GELO_F32 && dtype != GELO_BF16) return fail(ctx, GELO_EINVAL, "unknown dtype %d", (int)dtype);
    if (n < 1 || d < 1 || p < 1) return fail(ctx, GELO_EINVAL, "n=%d d=%d p=%d", n, d, p);
    if (d % 8 != 0 || p % 8 != 0) return fail(ctx, GELO_EALIGN, "d=%d and p=%d must be multiples of 8", d, p);
    gelo_status st = check_matrix(ctx, "U", U, ldu, d);
    if (st == GELO_OK) st = check_matrix(ctx, "W", W, ldw, p);
    if (st == GELO_OK) st = check_matrix(ctx, "Y", Y, ldy, p);
    if (st != GELO_OK) return st;
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    const size_t need = project_ws_need(dtype, n, d, p);
    if (need > 0) {
        st = grow(ctx, &ctx->project_ws, &ctx->project_ws_bytes, need);
        if (st != GELO_OK) return st;
    }
    return project_launch(ctx, dtype, n, d, p, U, ldu, W, ldw, Y, ldy, need > 0 ? ctx->project_ws : nullptr, need > 0 ? ctx->project_ws_bytes : 0,
                          (hipStream_t)stream);
}

gelo_status gelo_unmix(gelo_ctx* ctx, gelo_mixing* m, gelo_dtype dtype, int p, const void* Y, int64_t ldy,
                       void* Z, int64_t ldz, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or freed");
    if (dtype != GELO_F32 && dtype != GELO_BF16) return fail(ctx, GELO_EINVAL, "unknown dtype %d", (int)dtype);
    if ((int)dtype != m->dtype) return fail(ctx, GELO_EDTYPE, "Y and Z are %s but the mixing object was drawn for %s", dtype == GELO_BF16 ? "bf16" : "f32", m->dtype == GELO_BF16 ? "bf16" : "f32");
    if (p < 1) return fail(ctx, GELO_EINVAL, "p=%d", p);
    if (p % 8 != 0) return fail(ctx, GELO_EALIGN, "p=%d is not a multiple of 8", p);
    gelo_status st = check_matrix(ctx, "Y", Y, ldy, p);
    if (st == GELO_OK) st = check_matrix(ctx, "Z", Z, ldz, p);
    if (st != GELO_OK) return st;
    if (!ctx->allow_reuse && m->consumed) return fail(ctx, GELO_EREUSE, "this mixing object has already been consumed");
    if (!m->mixed) return fail(ctx, GELO_ESTATE, "gelo_unmix before gelo_mix");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    if (s != m->sample_stream) GELO_HIP(ctx, hipStreamWaitEvent(s, m->ready, 0));
    st = unmix_launch(ctx, m, p, Y, ldy, Z, ldz, s);
    if (st != GELO_OK) return st;
    m->consumed = true; m->last_stream = s;
    return GELO_OK;
}

gelo_status gelo_mixing_info(gelo_ctx* ctx, const gelo_mixing* m, int* n_data, int* k_shield, int* d,
                             gelo_dtype* dtype, gelo_kind* kind) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or freed");
    if (n_data) *n_data = m->n_data;
    if (k_shield) *k_shield = m->k;
    if (d) *d = m->d;
    if (dtype) *dtype = (gelo_dtype)m->dtype;
    if (kind) *kind = (gelo_kind)m->kind;
    return GELO_OK;
}

gelo_status gelo_sample_mixing_batch(gelo_ctx* ctx, gelo_kind kind, int n_data, int k_shield, int d, gelo_dtype dtype,
                                     uint64_t first_batch_id, int count, gelo_mixing** out, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!out) return fail(ctx, GELO_EINVAL, "out is NULL");
    if (count < 1 || count > GELO_MAX_BATCH_DRAW) return fail(ctx, GELO_EINVAL, "count=%d outside 1..%d", count, GELO_MAX_BATCH_DRAW);
    for (int i = 0; i < count; ++i) out[i] = nullptr;
    if (kind != GELO_ORTHOGONAL && kind != GELO_BLOCK_ORTHOGONAL && kind != GELO_REFLECTOR_PRODUCT)
        return fail(ctx, GELO_EINVAL, "batched draws exist for GELO_ORTHOGONAL, GELO_BLOCK_ORTHOGONAL and GELO_REFLECTOR_PRODUCT only");
    if (first_batch_id > UINT64_MAX - (uint64_t)count) return fail(ctx, GELO_EINVAL, "batch ids leave 64 bits");
    int n = 0;
    for (int i = 0; i < count; ++i) {
        gelo_status st = check_sample_args(ctx, kind, n_data, k_shield, d, dtype, 1.0, 1, first_batch_id + (uint64_t)i, &n);
        if (st != GELO_OK) return st;
    }
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const bool blocked = kind == GELO_BLOCK_ORTHOGONAL;
    const bool small = kind == GELO_ORTHOGONAL && n <= kSmallMaxN;
    // larger matrices: up to kQrSideBySide factorisations share every launch, each in a workspace of its own
    const size_t ws_bytes = up256(factor_workspace_bytes(n));
    const int side = qr_side_by_side(count, ws_bytes);
    gelo_status st = small ? GELO_OK : grow(ctx, &ctx->factor_ws, &ctx->factor_ws_bytes, blocked ? block_workspace_bytes(n) * count : ws_bytes * side);
    if (st != GELO_OK) return st;
    SmallSampleTargets t;
    gelo_mixing* got[GELO_MAX_BATCH_DRAW];
    int have = 0;
    for (int i = 0; i < count && st == GELO_OK; ++i) {
        gelo_mixing* m = nullptr;
        st = acquire_mixing(ctx, n_data, k_shield, d, dtype, form_of(kind), &m);
        if (st != GELO_OK) break;
        if (m->last_stream != nullptr || m->mixed) {
            hipError_t e = hipStreamWaitEvent(s, m->released, 0);
            if (e != hipSuccess) { st = hip_fail(ctx, e, "hipStreamWaitEvent"); break; }
        }
        m->in_use = true;                        // so that the next acquire takes another object
        got[have++] = m;
        t.block[i] = m->block;
    }
    PhiloxStream ps;
    ps.key0 = (uint32_t)ctx->seed; ps.key1 = (uint32_t)(ctx->seed >> 32);
    ps.c1 = kStreamMixing << 8; ps.c2 = ps.c3 = 0;
    if (st == GELO_OK && small) {
        small_targets_layout(got[0], &t);
        hipError_t e = small_sample(t, count, first_batch_id, ps, kStreamShield << 8, n, k_shield, d, got[0]->ldk, s);
        if (e != hipSuccess) st = hip_fail(ctx, e, "small_sample");
    }
    if (st == GELO_OK && blocked) {
        // all full blocks of all objects share the launches of ONE batched factorisation (workspaces: object-major,
        // then block), the last, shorter blocks of all objects those of a second one
        constexpr int B = GELO_BLOCK_ROWS;
        const int full = n / B, rest = n % B;
        const size_t wb = up256(factor_workspace_bytes(B)), wr = rest ? up256(factor_workspace_bytes(rest)) : 0;
        char* base_full = (char*)ctx->factor_ws;
        char* base_rest = base_full + wb * (size_t)full * count;
        hipError_t e = hipSuccess;
        FactorWorkspace w;
        for (int o = 0; o < count && e == hipSuccess; ++o) {
            const uint64_t id = first_batch_id + (uint64_t)o;
            ps.c2 = (uint32_t)id; ps.c3 = (uint32_t)(id >> 32);
            for (int i = 0; i < full && e == hipSuccess; ++i) {
                factor_workspace_carve(base_full + wb * ((size_t)o * full + i), B, &w);
                ps.c1 = (kStreamBlock << 8) | (uint32_t)i;
                e = fill_normal(w.M, w.n_pad / 16, B, B, ps, 1.0f, 1, s);
            }
            if (rest > 0 && e == hipSuccess) {
                factor_workspace_carve(base_rest + wr * o, rest, &w);
                ps.c1 = (kStreamBlock << 8) | (uint32_t)full;
                e = fill_normal(w.M, w.n_pad / 16, rest, rest, ps, 1.0f, 1, s);
            }
        }
        if (full > 0 && e == hipSuccess) {
            factor_workspace_carve(base_full, B, &w);
            e = householder_qr(w, B, full * count, (int64_t)(wb / sizeof(float)), s);
        }
        if (rest > 0 && e == hipSuccess) {
            factor_workspace_carve(base_rest, rest, &w);
            e = householder_qr(w, rest, count, (int64_t)(wr / sizeof(float)), s);
        }
        for (int o = 0; o < count && e == hipSuccess; ++o) {
            gelo_mixing* m = got[o];
            const uint64_t id = first_batch_id + (uint64_t)o;
            for (int i = 0; i < full + (rest ? 1 : 0) && e == hipSuccess; ++i) {
                const int rows = i < full ? B : rest;
                if (i < full) factor_workspace_carve(base_full + wb * ((size_t)o * full + i), B, &w);
                else factor_workspace_carve(base_rest + wr * o, rest, &w);
                const int64_t at = (int64_t)i * B * m->ldk;
                e = emit_matrix(w.X, w.n_pad / 16, 1, w.rdiag, rows, m->ldk, m->A32 + at, m->A16 ? m->A16 + at : nullptr,
                                m->Ainv32 + at, m->Ainv16 ? m->Ainv16 + at : nullptr, s);
            }
            if (e == hipSuccess && k_shield > 0) {
                ps.c1 = kStreamShield << 8; ps.c2 = (uint32_t)id; ps.c3 = (uint32_t)(id >> 32);
                e = shield_directions(m->GS, k_shield, d, ps, m->gsnorm, s);
            }
        }
        if (e != hipSuccess) st = hip_fail(ctx, e, "batched block-orthogonal draw");
    }
    for (int base = 0; st == GELO_OK && !small && !blocked && base < count; base += side) {
        const int c = count - base < side ? count - base : side;
        FactorWorkspace lw[kQrSideBySide];
        hipError_t e = hipSuccess;
        for (int i = 0; i < c && e == hipSuccess; ++i) {
            factor_workspace_carve((char*)ctx->factor_ws + ws_bytes * i, n, &lw[i]);
            const uint64_t id = first_batch_id + (uint64_t)(base + i);
            ps.c1 = kStreamMixing << 8; ps.c2 = (uint32_t)id; ps.c3 = (uint32_t)(id >> 32);
            e = fill_normal(lw[i].M, lw[i].n_pad / 16, n, n, ps, 1.0f, kind == GELO_REFLECTOR_PRODUCT ? 2 : 1, s);      // straight into the QR's tiles
        }
        if (e == hipSuccess) e = householder_qr(lw[0], n, c, (int64_t)(ws_bytes / sizeof(float)), s, kind == GELO_REFLECTOR_PRODUCT);
        for (int i = 0; i < c && e == hipSuccess; ++i) {
            gelo_mixing* m = got[base + i];
            const uint64_t id = first_batch_id + (uint64_t)(base + i);
            // A = Q diag(sign r_ii); A^-1 = A^T
            e = emit_matrix(lw[i].X, lw[i].n_pad / 16, 1, lw[i].rdiag, n, m->ldk, m->A32, m->A16, m->Ainv32, m->Ainv16, s);
            if (e == hipSuccess && k_shield > 0) {
                ps.c1 = kStreamShield << 8; ps.c2 = (uint32_t)id; ps.c3 = (uint32_t)(id >> 32);
                e = shield_directions(m->GS, k_shield, d, ps, m->gsnorm, s);
            }
        }
        if (e != hipSuccess) st = hip_fail(ctx, e, "batched orthogonal draw");
    }
    if (st != GELO_OK) {
        for (int i = 0; i < have; ++i) got[i]->in_use = false;
        return st;
    }
    for (int i = 0; i < count; ++i) {
        gelo_mixing* m = got[i];
        m->kind = kind; m->attempt = 0; m->kappa = 1.0f; m->batch_id = first_batch_id + (uint64_t)i;
        m->mixed = false; m->consumed = false; m->sample_stream = s; m->last_stream = s;
        hipError_t e = hipEventRecord(m->ready, s);
        if (e != hipSuccess) return hip_fail(ctx, e, "hipEventRecord");
        batch_commit(ctx, m->batch_id);
        out[i] = m;
    }
    return GELO_OK;
}

gelo_status gelo_chain(gelo_ctx* ctx, gelo_mixing* m, gelo_dtype dtype, int p, const void* H, const void* W, float shield_scale,
                       gelo_norm_stat stat, void* Z, void* U, void* Y, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or freed");
    if (!U || !Y) return fail(ctx, GELO_EINVAL, "U and Y must not be NULL");
    gelo_status st = gelo_mix(ctx, m, dtype, H, m->d, shield_scale, stat, U, m->d, stream);
    if (st == GELO_OK) st = gelo_project(ctx, dtype, m->n, m->d, p, U, m->d, W, p, Y, p, stream);
    if (st == GELO_OK) st = gelo_unmix(ctx, m, dtype, p, Y, p, Z, p, stream);
    return st;
}

gelo_status gelo_mixing_free(gelo_ctx* ctx, gelo_mixing* m) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or already freed");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    GELO_HIP(ctx, hipEventRecord(m->released, m->last_stream));
    m->in_use = false;
    return GELO_OK;
}

gelo_status gelo_qkv_forward(gelo_ctx* ctx, gelo_kind kind, gelo_dtype dtype, int n_data, int k_shield,
                             int d, int p, const void* H, const void* W, float shield_scale,
                             gelo_norm_stat stat, double cond_max, int max_attempts, uint64_t batch_id,
                             void* Z, void* U_opt, void* Y_opt, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!H || !W || !Z) return fail(ctx, GELO_EINVAL, "H, W and Z must not be NULL");
    if (p < 1 || p % 8 != 0) return fail(ctx, p < 1 ? GELO_EINVAL : GELO_EALIGN, "p=%d must be a positive multiple of 8", p);
    if (dtype != GELO_F32 && dtype != GELO_BF16) return fail(ctx, GELO_EINVAL, "unknown dtype %d", (int)dtype);
    if (n_data < 1 || k_shield < 0 || d < 1) return fail(ctx, GELO_EINVAL, "n_data=%d k_shield=%d d=%d", n_data, k_shield, d);
    if (!aligned16(H) || !aligned16(W) || !aligned16(Z) || !aligned16(U_opt) || !aligned16(Y_opt))
        return fail(ctx, GELO_EALIGN, "H, W, Z, U and Y must be 16-byte aligned");
    const int64_t n = (int64_t)n_data + k_shield;
    void* U = U_opt; void* Y = Y_opt;
    if (!U || !Y) {
        GELO_HIP(ctx, hipSetDevice(ctx->device));
        const size_t ub = up256((size_t)n * d * elem_size(dtype)), yb = up256((size_t)n * p * elem_size(dtype));
        gelo_status st = grow(ctx, &ctx->chain_ws, &ctx->chain_ws_bytes, ub + yb);
        if (st != GELO_OK) return st;
        if (!U) U = ctx->chain_ws;
        if (!Y) Y = (char*)ctx->chain_ws + ub;
    }
    gelo_mixing* m = nullptr;
    gelo_status st = gelo_sample_mixing(ctx, kind, n_data, k_shield, d, dtype, cond_max, max_attempts, batch_id, &m, stream);
    if (st != GELO_OK) return st;
    st = gelo_mix(ctx, m, dtype, H, d, shield_scale, stat, U, d, stream);
    if (st == GELO_OK) st = gelo_project(ctx, dtype, (int)n, d, p, U, d, W, p, Y, p, stream);
    if (st == GELO_OK) st = gelo_unmix(ctx, m, dtype, p, Y, p, Z, p, stream);
    const std::string keep = ctx->err;
    gelo_mixing_free(ctx, m);
    if (st != GELO_OK) ctx->err = keep;
    return st;
}

gelo_status gelo_mixing_export(gelo_ctx* ctx, const gelo_mixing* m, float* A, float* A_inv,
                               float* S, int* attempt, float* kappa, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or freed");
    if (S && m->k > 0 && !m->mixed) return fail(ctx, GELO_ESTATE, "shield rows exist only after gelo_mix");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    if (s != m->sample_stream) GELO_HIP(ctx, hipStreamWaitEvent(s, m->ready, 0));
    if (m->structured && (A || A_inv)) {
        // the dense matrices exist only here: A = (the transform applied to the identity), in float
        const int64_t ldn = round_up(m->n, 8);
        const size_t mat = up256((size_t)m->n * ldn * 4);
        gelo_status st = grow(ctx, &ctx->chain_ws, &ctx->chain_ws_bytes, 2 * mat);
        if (st != GELO_OK) return st;
        float* eye = (float*)ctx->chain_ws;
        float* res = (float*)((char*)ctx->chain_ws + mat);
        GELO_HIP(ctx, set_identity(eye, ldn, m->n, s));
        for (int t = 0; t < 2; ++t) {
            float* dst = t == 0 ? A : A_inv;
            if (!dst) continue;
            StructuredOperands o;
            o.in0 = eye; o.ld0 = ldn; o.rows0 = m->n; o.in1 = nullptr; o.ld1 = 0;
            o.out = res; o.ldo = ldn; o.rows_out = m->n;
            o.table = m->table; o.n = m->n; o.ncols = (int)ldn; o.rounds = kStructuredRounds; o.transposed = t == 1;
            GELO_HIP(ctx, structured_apply(o, 0, s));
            GELO_HIP(ctx, export_dense(res, 0, ldn, m->n, m->n, dst, s));
        }
    } else if (m->blocked) {
        // the dense n x n matrix that acts on the stacked [H; S]: block i's columns are its data rows' and,
        // behind column n_data, its shield rows'; A^-1 is the transpose
        const size_t row = (size_t)m->n * sizeof(float);
        if (A) GELO_HIP(ctx, hipMemsetAsync(A, 0, row * m->n, s));
        if (A_inv) GELO_HIP(ctx, hipMemsetAsync(A_inv, 0, row * m->n, s));
        for (int i = 0; i < block_count(m->n); ++i) {
            const BlockPiece b = block_piece(m->n_data, m->k, i);
            const float* Ai = m->A32 + (int64_t)b.row0 * m->ldk;
            const float* Ti = m->Ainv32 + (int64_t)b.row0 * m->ldk;
            const size_t pitch = (size_t)m->ldk * sizeof(float);
            if (A && b.data_rows > 0)
                GELO_HIP(ctx, hipMemcpy2DAsync(A + (int64_t)b.row0 * m->n + b.data0, row, Ai, pitch, b.data_rows * sizeof(float), b.rows, hipMemcpyDeviceToDevice, s));
            if (A && b.shield_rows > 0)
                GELO_HIP(ctx, hipMemcpy2DAsync(A + (int64_t)b.row0 * m->n + m->n_data + b.shield0, row, Ai + b.data_rows, pitch, b.shield_rows * sizeof(float), b.rows, hipMemcpyDeviceToDevice, s));
            if (A_inv && b.data_rows > 0)
                GELO_HIP(ctx, hipMemcpy2DAsync(A_inv + (int64_t)b.data0 * m->n + b.row0, row, Ti, pitch, b.rows * sizeof(float), b.data_rows, hipMemcpyDeviceToDevice, s));
            if (A_inv && b.shield_rows > 0)
                GELO_HIP(ctx, hipMemcpy2DAsync(A_inv + (int64_t)(m->n_data + b.shield0) * m->n + b.row0, row, Ti + (int64_t)b.data_rows * m->ldk, pitch, b.rows * sizeof(float), b.shield_rows, hipMemcpyDeviceToDevice, s));
        }
    } else {
        if (A) GELO_HIP(ctx, export_dense(m->A32, 0, m->ldk, m->n, m->n, A, s));
        if (A_inv) GELO_HIP(ctx, export_dense(m->Ainv32, 0, m->ldk, m->n, m->n, A_inv, s));
    }
    if (S && m->k > 0) GELO_HIP(ctx, export_dense(m->S, m->dtype == GELO_BF16, m->d, m->k, m->d, S, s));
    if (attempt) *attempt = m->attempt;
    if (kappa) {
        if (m->kappa < 0.f) {
            GELO_HIP(ctx, hipMemcpyAsync(ctx->host_scalars, m->stat + 1, sizeof(float), hipMemcpyDeviceToHost, s));
            GELO_HIP(ctx, hipStreamSynchronize(s));
            *kappa = ctx->host_scalars[0];
        } else {
            *kappa = m->kappa;
        }
    }
    return GELO_OK;
}

gelo_status gelo_qkv_forward_static(gelo_ctx* ctx, gelo_kind kind, gelo_dtype dtype, int n_data, int k_shield,
                                    int d, int p, const void* H, const void* W, float shield_scale,
                                    gelo_norm_stat stat, uint64_t batch_id, void* Z, void* U, void* Y, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!H || !W || !Z || !U || !Y) return fail(ctx, GELO_EINVAL, "H, W, Z, U and Y must not be NULL");
    if (!aligned16(H) || !aligned16(W) || !aligned16(Z) || !aligned16(U) || !aligned16(Y))
        return fail(ctx, GELO_EALIGN, "H, W, Z, U and Y must be 16-byte aligned");
    if (p < 1 || p % 8 != 0) return fail(ctx, p < 1 ? GELO_EINVAL : GELO_EALIGN, "p=%d must be a positive multiple of 8", p);
    if (kind == GELO_GAUSSIAN) return fail(ctx, GELO_EINVAL, "GELO_GAUSSIAN reads condition estimates back and uses buffers of its own: not available without allocation");
    if (stat != GELO_NORM_MEDIAN && stat != GELO_NORM_MEAN) return fail(ctx, GELO_EINVAL, "unknown norm statistic %d", (int)stat);
    if (k_shield > 0 && !(shield_scale > 0.f)) return fail(ctx, GELO_EINVAL, "shield_scale=%g must be positive", (double)shield_scale);
    int n = 0;
    gelo_status st = check_sample_args(ctx, kind, n_data, k_shield, d, dtype, 1.0, 1, batch_id, &n);
    if (st != GELO_OK) return st;
    const bool structured = kind == GELO_STRUCTURED;
    if (n > GELO_STATIC_MAX_N) return fail(ctx, GELO_ESHAPE, "n = %d exceeds GELO_STATIC_MAX_N = %d", n, GELO_STATIC_MAX_N);
    const MixingLayout L = mixing_layout(n_data, k_shield, d, dtype, form_of(kind));
    const size_t ws_bytes = structured ? 0 : kind == GELO_BLOCK_ORTHOGONAL ? block_workspace_bytes(n) : up256(factor_workspace_bytes(n));
    if (L.total + ws_bytes > kStaticScratchBytes)
        return fail(ctx, GELO_ESHAPE, "this batch needs %zu bytes of scratch, the static buffer holds %zu (n <= %d, and k_shield * d bounded by it)",
                    L.total + ws_bytes, kStaticScratchBytes, GELO_STATIC_MAX_N);
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    // the mixing object of this call lives on the host stack and points into the static device array
    gelo_mixing local = {};
    char* base = (char*)ctx->static_scratch;
    carve_mixing(&local, base, n_data, k_shield, d, dtype, form_of(kind));
    FactorWorkspace ws = {};
    if (kind == GELO_BLOCK_ORTHOGONAL) ws.M = (float*)(base + up256(L.total));      // sample_into carves the blocks' workspaces from here
    else if (!structured) factor_workspace_carve(base + up256(L.total), n, &ws);
    st = sample_into(ctx, &local, ws, ws_bytes, 1, kind, 1.0, 1, batch_id, s);
    if (st == GELO_OK) batch_commit(ctx, batch_id);
    if (st == GELO_OK) st = mix_launch(ctx, &local, H, d, shield_scale, stat, U, d, s);
    // partial sums of the projection: behind the batch's buffers if the static array still holds them (else K is not cut)
    const size_t used = up256(L.total) + ws_bytes;
    const size_t need = project_ws_need(dtype, n, d, p);
    const bool fits = need > 0 && used + need <= kStaticScratchBytes;
    if (st == GELO_OK) st = project_launch(ctx, dtype, n, d, p, U, d, W, p, Y, p, fits ? base + used : nullptr, fits ? need : 0, s);
    if (st == GELO_OK) st = unmix_launch(ctx, &local, p, Y, p, Z, p, s);
    return st;
}

gelo_status gelo_reserve(gelo_ctx* ctx, gelo_kind kind, gelo_dtype dtype, int n_data, int k_shield, int d, int p,
                         int max_attempts, int mixings) {
    if (!ctx) return GELO_EINVAL;
    if (mixings < 0 || p < 0) return fail(ctx, GELO_EINVAL, "mixings=%d p=%d", mixings, p);
    int n = 0;
    const bool reuse = ctx->allow_reuse;
    ctx->allow_reuse = true;                    // no batch id is involved here
    gelo_status st = check_sample_args(ctx, kind, n_data, k_shield, d, dtype, 1.0, kind == GELO_GAUSSIAN ? max_attempts : 1, 0, &n);
    ctx->allow_reuse = reuse;
    if (st != GELO_OK) return st;
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    int lanes = 1;
    st = prepare_sampling(ctx, kind, n, dtype, max_attempts, &lanes);
    if (st != GELO_OK) return st;
    if (kind == GELO_BLOCK_ORTHOGONAL && mixings > 1) {
        st = grow(ctx, &ctx->factor_ws, &ctx->factor_ws_bytes, block_workspace_bytes(n) * (mixings < GELO_MAX_BATCH_DRAW ? mixings : GELO_MAX_BATCH_DRAW));
        if (st != GELO_OK) return st;
    }
    if (((kind == GELO_ORTHOGONAL && n > kSmallMaxN) || kind == GELO_REFLECTOR_PRODUCT) && mixings > 1) {
        // a batched draw of `mixings` matrices factorises up to kQrSideBySide of them side by side
        const int side = qr_side_by_side(mixings, up256(factor_workspace_bytes(n)));
        st = grow(ctx, &ctx->factor_ws, &ctx->factor_ws_bytes, up256(factor_workspace_bytes(n)) * side);
        if (st != GELO_OK) return st;
    }
    if (p > 0) {
        const size_t ub = up256((size_t)n * d * elem_size(dtype)), yb = up256((size_t)n * p * elem_size(dtype));
        st = grow(ctx, &ctx->chain_ws, &ctx->chain_ws_bytes, ub + yb);
        if (st != GELO_OK) return st;
        const size_t need = project_ws_need(dtype, n, d, p);
        if (need > 0) st = grow(ctx, &ctx->project_ws, &ctx->project_ws_bytes, need);
        if (st != GELO_OK) return st;
    }
    // `mixings` free objects of this shape in the pool
    std::vector<gelo_mixing*> got;
    for (int i = 0; i < mixings && st == GELO_OK; ++i) {
        gelo_mixing* m = nullptr;
        st = acquire_mixing(ctx, n_data, k_shield, d, dtype, form_of(kind), &m);
        if (st == GELO_OK) { m->in_use = true; got.push_back(m); }
    }
    for (gelo_mixing* m : got) m->in_use = false;
    return st;
}

gelo_status gelo_set_batch_floor(gelo_ctx* ctx, uint64_t first_unused) {
    if (!ctx) return GELO_EINVAL;
    if (first_unused < ctx->batch_floor) return fail(ctx, GELO_EINVAL, "the floor only moves up (it is %llu)", (unsigned long long)ctx->batch_floor);
    ctx->batch_floor = first_unused;
    return GELO_OK;
}

gelo_status gelo_get_batch_floor(const gelo_ctx* ctx, uint64_t* first_unused) {
    if (!ctx || !first_unused) return GELO_EINVAL;
    *first_unused = ctx->batch_high > ctx->batch_floor ? ctx->batch_high : ctx->batch_floor;
    return GELO_OK;
}

gelo_status gelo_debug_philox_words(gelo_ctx* ctx, uint32_t stream_id, uint32_t attempt, uint64_t batch_id,
                                    uint32_t first_block, uint32_t blocks, uint32_t* words, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!words || (reinterpret_cast<uintptr_t>(words) & 15u)) return fail(ctx, words ? GELO_EALIGN : GELO_EINVAL, "words must be a 16-byte aligned device pointer");
    if (stream_id > 0xFFFFFFu || attempt > 255u) return fail(ctx, GELO_EINVAL, "stream_id=%u attempt=%u", stream_id, attempt);
    if ((uint64_t)first_block + blocks > ((uint64_t)1 << 32)) return fail(ctx, GELO_EINVAL, "block range leaves 32 bits");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    PhiloxStream ps;
    ps.key0 = (uint32_t)ctx->seed; ps.key1 = (uint32_t)(ctx->seed >> 32);
    ps.c1 = (stream_id << 8) | attempt; ps.c2 = (uint32_t)batch_id; ps.c3 = (uint32_t)(batch_id >> 32);
    GELO_HIP(ctx, philox_words(words, first_block, blocks, ps, (hipStream_t)stream));
    return GELO_OK;
}

gelo_status gelo_mixing_export_table(gelo_ctx* ctx, const gelo_mixing* m, uint32_t* table, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!m || !owns(ctx, m) || !m->in_use) return fail(ctx, GELO_EINVAL, "mixing object is NULL, foreign or freed");
    if (!m->structured) return fail(ctx, GELO_EINVAL, "only a GELO_STRUCTURED mixing object has a table");
    if (!table) return fail(ctx, GELO_EINVAL, "table is NULL");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    if (s != m->sample_stream) GELO_HIP(ctx, hipStreamWaitEvent(s, m->ready, 0));
    // the library's tables start on 16-byte boundaries; the caller's are packed
    GELO_HIP(ctx, hipMemcpy2DAsync(table, (size_t)m->n * sizeof(uint32_t), m->table, (size_t)round_up(m->n, 4) * sizeof(uint32_t),
                                   (size_t)m->n * sizeof(uint32_t), kStructuredRounds + 1, hipMemcpyDeviceToDevice, s));
    return GELO_OK;
}

gelo_status gelo_fp8_weight_bytes(int d, int p, size_t* bytes) {
    if (!bytes || d < 1 || p < 1) return GELO_EINVAL;
    *bytes = up256((size_t)p * d) + (size_t)p * sizeof(float);
    return GELO_OK;
}

static gelo_status check_fp8_shape(gelo_ctx* ctx, int d, int p) {
    if (d < 1 || p < 1) return fail(ctx, GELO_EINVAL, "d=%d p=%d", d, p);
    if (d % 128 != 0) return fail(ctx, GELO_ESHAPE, "the 8-bit projection takes d a multiple of 128 (d = %d)", d);
    if (p % 8 != 0) return fail(ctx, GELO_EALIGN, "p=%d is not a multiple of 8", p);
    return GELO_OK;
}

gelo_status gelo_prepare_weight_fp8(gelo_ctx* ctx, int d, int p, const void* W, int64_t ldw, void* Wq, void* stream) {
    if (!ctx) return GELO_EINVAL;
    gelo_status st = check_fp8_shape(ctx, d, p);
    if (st == GELO_OK) st = check_matrix(ctx, "W", W, ldw, p);
    if (st != GELO_OK) return st;
    if (!Wq || !aligned16(Wq)) return fail(ctx, Wq ? GELO_EALIGN : GELO_EINVAL, "Wq must be a 16-byte aligned device buffer");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    uint8_t* codes = (uint8_t*)Wq;
    float* scale = (float*)(codes + up256((size_t)p * d));
    GELO_HIP(ctx, quantize_weight_e4m3(W, ldw, d, p, codes, scale, (hipStream_t)stream));
    return GELO_OK;
}

gelo_status gelo_project_fp8(gelo_ctx* ctx, int n, int d, int p, const void* U, int64_t ldu, const void* Wq,
                             void* Y, int64_t ldy, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (n < 1) return fail(ctx, GELO_EINVAL, "n=%d", n);
    gelo_status st = check_fp8_shape(ctx, d, p);
    if (st == GELO_OK) st = check_matrix(ctx, "U", U, ldu, d);
    if (st == GELO_OK) st = check_matrix(ctx, "Y", Y, ldy, p);
    if (st != GELO_OK) return st;
    if (!Wq || !aligned16(Wq)) return fail(ctx, Wq ? GELO_EALIGN : GELO_EINVAL, "Wq must be a 16-byte aligned device buffer");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    const size_t code_bytes = up256((size_t)n * d);
    st = grow(ctx, &ctx->quant_ws, &ctx->quant_ws_bytes, code_bytes + up256((size_t)n * sizeof(float)));
    if (st != GELO_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    uint8_t* ucodes = (uint8_t*)ctx->quant_ws;
    float* uscale = (float*)(ucodes + code_bytes);
    const uint8_t* wcodes = (const uint8_t*)Wq;
    const float* wscale = (const float*)(wcodes + up256((size_t)p * d));
    GELO_HIP(ctx, quantize_rows_e4m3(U, ldu, n, d, ucodes, d, uscale, s));
    GELO_HIP(ctx, gemm_fp8(ucodes, d, uscale, wcodes, d, wscale, Y, ldy, n, p, d, s));
    return GELO_OK;
}

gelo_status gelo_debug_quantize_rows_fp8(gelo_ctx* ctx, int n, int d, const void* U, int64_t ldu, uint8_t* codes,
                                         float* scales, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (n < 1 || d < 8 || d % 8 != 0) return fail(ctx, GELO_EINVAL, "n=%d d=%d", n, d);
    gelo_status st = check_matrix(ctx, "U", U, ldu, d);
    if (st != GELO_OK) return st;
    if (!codes || !scales || !aligned16(codes)) return fail(ctx, GELO_EINVAL, "codes (16-byte aligned) and scales must be device buffers");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    GELO_HIP(ctx, quantize_rows_e4m3(U, ldu, n, d, codes, d, scales, (hipStream_t)stream));
    return GELO_OK;
}

gelo_status gelo_measure_matrix_rate(gelo_ctx* ctx, int fp8, int iters, int launches, double* seconds, double* flop, void* stream) {
    if (!ctx) return GELO_EINVAL;
    if (!seconds || !flop) return fail(ctx, GELO_EINVAL, "seconds and flop must not be NULL");
    if (iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1000 || (fp8 != 0 && fp8 != 1))
        return fail(ctx, GELO_EINVAL, "fp8=%d iters=%d launches=%d", fp8, iters, launches);
    if (!ctx->static_scratch || matrix_rate_scratch_bytes() > kStaticScratchBytes) return fail(ctx, GELO_ESTATE, "no scratch buffer on this device");
    GELO_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    GELO_HIP(ctx, hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    double f = 0.0;
    if (e == hipSuccess) e = matrix_rate_launch(fp8, iters, (float*)ctx->static_scratch, &f, s);      // clocks settle under the load
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    for (int i = 0; i < launches && e == hipSuccess; ++i) e = matrix_rate_launch(fp8, iters, (float*)ctx->static_scratch, &f, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(ctx, e, "matrix rate measurement");
    *seconds = (double)ms * 1e-3 / launches;
    *flop = f;
    return GELO_OK;
}

}  // extern "C"
