// Host side of the C ABI declared in include/w2v.h: argument validation, the host-built sampling
// table and subsampling thresholds, kernel launches, the host-fed batch loop.  No device memory is
// allocated here: tables and accumulators live in the caller's workspace, staging in the caller's buffer.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <functional>
#include <new>
#include <vector>

#include "w2v_internal.h"
#include "w2v_rng.h"

namespace w2v {

static uint64_t align256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

WorkspaceLayout workspace_layout(uint32_t vocab, uint32_t table_size, uint64_t snap_bytes)
{
    WorkspaceLayout l;
    l.accum_off = 0;
    l.thr_off = align256(sizeof(Accum));
    l.snap_off = l.thr_off + align256((uint64_t)vocab * sizeof(uint32_t));
    l.table_off = l.snap_off + align256(snap_bytes);
    l.total = l.table_off + align256((uint64_t)table_size * sizeof(int32_t));
    return l;
}

}  // namespace w2v

static_assert(sizeof(w2v::Accum) <= 256, "the accumulator block heads the static scratch array");

namespace {

std::string g_create_error;

int fail(w2v_ctx *ctx, int code, const std::string &msg)
{
    if (ctx) ctx->err = msg; else g_create_error = msg;
    return code;
}

int fail_hip(w2v_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, W2V_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define HIP_TRY(ctx, expr)                                         \
    do {                                                           \
        hipError_t e_ = (expr);                                    \
        if (e_ != hipSuccess) return fail_hip((ctx), e_, #expr);   \
    } while (0)

// returns an empty string when cfg is acceptable
std::string check_config(const w2v_config *c)
{
    if (!c) return "cfg is NULL";
    if (c->struct_size != sizeof(w2v_config)) return "cfg.struct_size does not match sizeof(w2v_config)";
    if (c->vocab < 1 || c->vocab > W2V_MAX_VOCAB) return "cfg.vocab out of range [1, 2^27]";
    if (c->dim < 1 || c->dim > W2V_MAX_DIM) return "cfg.dim out of range [1, 512]";
    if (c->window < 1 || c->window > W2V_MAX_WINDOW) return "cfg.window out of range [1, 16]";
    if (c->negatives > W2V_MAX_NEGATIVES) return "cfg.negatives out of range [0, 20]";
    if (c->window_mode > 1) return "cfg.window_mode must be 0 or 1";
    if (c->negative_block > 64u || (c->negative_block & (c->negative_block - 1u)) != 0)
        return "cfg.negative_block must be 0 or a power of two up to 64";
    if (c->update_mode > 2) return "cfg.update_mode must be 0 (automatic), 1 (overwrite) or 2 (summed)";
    if (c->storage > 1) return "cfg.storage must be 0 (float) or 1 (bfloat16)";
    if (c->storage == 1 && c->update_mode == 2) return "cfg.storage 1 (bfloat16 tables) always overwrites: cfg.update_mode must be 0 or 1";
    if (c->reserved != 0) return "cfg.reserved must be 0";
    if (c->total_epochs < 1) return "cfg.total_epochs must be >= 1";
    if (c->tokens_per_epoch < 1) return "cfg.tokens_per_epoch must be >= 1";
    if (c->tokens_per_epoch > (1ull << 52) / c->total_epochs) return "total_epochs * tokens_per_epoch exceeds 2^52";
    if (!(c->lr0 > 0.0) || !std::isfinite(c->lr0)) return "cfg.lr0 must be positive and finite";
    if (!(c->lr_min_frac >= 0.0) || c->lr_min_frac > 1.0) return "cfg.lr_min_frac must be in [0, 1]";
    if (!(c->subsample_t >= 0.0) || !std::isfinite(c->subsample_t)) return "cfg.subsample_t must be >= 0";
    if (!c->syn0 || !c->syn1neg) return "cfg.syn0 / cfg.syn1neg is NULL";
    if (c->ld < c->dim || (c->ld % 4u) != 0) return "cfg.ld must be >= dim and a multiple of 4";
    if (c->device < 0) return "cfg.device must be >= 0";
    if (!c->workspace) return "cfg.workspace is NULL";
    if (((uintptr_t)c->workspace & 255u) != 0) return "cfg.workspace must be 256-byte aligned";
    w2v::RowShape s;
    if (!w2v::pick_row_shape(c->dim, c->ld, &s)) return "cfg.dim: no lane layout for this dimension";
    const uint32_t span = c->window_mode ? (c->window + 1u) / 2u : c->window;      // widest window that occurs
    if ((uint32_t)(64 * w2v::floats_per_lane(s)) * span > 512u * 10u)
        return "cfg.dim * cfg.window too large (rows of more than 320 floats need window <= 10)";
    return std::string();
}

w2v::KernelArgs kernel_args(const w2v_ctx *ctx, const int32_t *tokens, const uint64_t *sent_off, uint64_t n_sent,
                            uint64_t first_pos, uint32_t epoch)
{
    const w2v_config &c = ctx->cfg;
    unsigned char *ws = static_cast<unsigned char *>(c.workspace);
    w2v::KernelArgs a;
    std::memset(&a, 0, sizeof(a));
    a.syn0 = static_cast<float *>(c.syn0);
    a.syn1neg = static_cast<float *>(c.syn1neg);
    a.tokens = tokens;
    a.sent_off = sent_off;
    a.table = reinterpret_cast<const int32_t *>(ws + ctx->ws.table_off);
    a.thr = reinterpret_cast<const uint32_t *>(ws + ctx->ws.thr_off);
    a.accum = reinterpret_cast<w2v::Accum *>(ws + ctx->ws.accum_off);
    a.n_sent = n_sent;
    a.first_pos = first_pos;
    a.key = w2v::epoch_key(c.seed, epoch);
    a.lr_done_base = (uint64_t)epoch * c.tokens_per_epoch;
    a.lr_all = (uint64_t)c.total_epochs * c.tokens_per_epoch;
    a.lr0 = c.lr0;
    a.lr_min_frac = c.lr_min_frac;
    a.vocab = c.vocab;
    a.dim = c.dim;
    a.ld = c.ld;
    // fixed width ceil(W/2): the kernels see that width as their window, so the ring holds 2*ceil(W/2)+2 rows
    a.window = c.window_mode ? (c.window + 1u) / 2u : c.window;
    a.negatives = c.negatives;
    a.window_mode = c.window_mode ? 2u : 0u;
    a.table_size = ctx->table_size;
    a.subsample = c.subsample_t > 0.0 ? 1u : 0u;
    a.neg_shift = 0;
    for (uint32_t b = c.negative_block; b > 1u; b >>= 1) ++a.neg_shift;
    return a;
}

int check_train_call(w2v_ctx *ctx, const int32_t *tokens, const uint64_t *sent_off, uint64_t n_sent,
                     uint64_t first_pos, uint32_t epoch)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    if (!ctx->table_built) return fail(ctx, W2V_ESTATE, "w2v_build_unigram_table must be called first");
    if (epoch >= ctx->cfg.total_epochs) return fail(ctx, W2V_EINVAL, "epoch must be < cfg.total_epochs");
    if (first_pos > ctx->cfg.tokens_per_epoch) return fail(ctx, W2V_EINVAL, "first_token_global_pos exceeds cfg.tokens_per_epoch");
    if (n_sent && (!tokens || !sent_off)) return fail(ctx, W2V_EINVAL, "tokens / sent_off is NULL");
    return W2V_OK;
}

hipStream_t stream_of(const w2v_ctx *ctx) { return static_cast<hipStream_t>(ctx->cfg.stream); }

// Wavefronts for cfg.sentences_in_flight = 0: all the GPU holds, but no more than one per 2,048 * ((N+1)/6)^2 kept
// tokens of the epoch (one per 2,048 with five negatives).  Every wavefront trains on copies of the rows it touches
// and the last writer of a row wins: the chance that an update of a row is lost grows with the output rows in
// flight, wavefronts x (N+1), a window is spoilt if any of its N+1 rows is, and the updates a row gets per epoch
// grow with the tokens that survive subsampling.  Measured: a 3M-token corpus (N=5, half the tokens kept) on 3,000
// wavefronts reaches planted-cluster score 0.56 in five epochs, on 730 it reaches 1.00; a 0.6M-token corpus on 2,400
// wavefronts does not learn at all; 9.5M tokens of which 30 % are kept, N=10, on 1,536 wavefronts: score 0.67 after
// two epochs, on 512: 1.00; 5.6M tokens of that kind, four epochs, loss against the serial oracle: 360 wavefronts
// +0.9 %, 196 (this rule) +0.6 %.  The 17M-token corpus (N=5) keeps every wavefront.
//
// Summed updates lose nothing, but every change is made to a copy that does not see what the other holders of the row
// do meanwhile, and the changes of all holders add up: where many wavefronts hold one row at once the step on that row
// multiplies and the loss ends higher.  The measure is the collision mass C = wavefronts x rows a wavefront holds
// (2W+2 ring rows + N+1 output rows) x sum over words of (share of the kept tokens)^2, the expected number of other
// wavefronts that hold the row of a token at the moment it is used.  Measured on uniform walks (W=10, N=5, two
// epochs, loss against strict order): 100,000 nodes, 16M tokens: C=2.2 (2,304 wavefronts) +2.2 %, C=0.49 (512)
// +0.44 %; 100,000 nodes, 80M tokens: C=2.2 +1.5 %, C=0.98 +0.9 %, C=0.49 +0.5 %, C=0.24 +0.2 %; 1M nodes, 80M
// tokens: C=0.27 (all 2,304 wavefronts) +0.5 %.  The summed mode therefore runs at most 0.5 / (rows x mass) wavefronts.
uint64_t lock_free_waves(const w2v_ctx *ctx, uint64_t resident, int update)
{
    const double kept = (double)ctx->cfg.tokens_per_epoch * ctx->kept_fraction;
    const double rows = (double)(ctx->cfg.negatives + 1u);
    uint64_t cap = (uint64_t)(kept * 36.0 / (2048.0 * rows * rows));
    if (update == 1 && ctx->collision_mass > 0.0) {
        const uint32_t w = ctx->cfg.window_mode ? (ctx->cfg.window + 1u) / 2u : ctx->cfg.window;
        const double held = (double)(2u * w + 2u) + rows;
        const double by_mass = 0.5 / (held * ctx->collision_mass);
        if (by_mass < (double)cap) cap = (uint64_t)by_mass;
    }
    if (cap < 64u) cap = 64u;
    return resident < cap ? resident : cap;
}

// Bytes of snapshot space in the workspace: the summed mode keeps the starting value of every ring slot of every
// wavefront there.  None when the configuration rules the mode out or no such kernel exists for its shape.
uint64_t snapshot_bytes(const w2v_config *c, uint32_t *floats_per_wave)
{
    *floats_per_wave = 0;
    if (c->update_mode == 1u || c->storage != 0u) return 0;
    w2v::KernelArgs a;
    std::memset(&a, 0, sizeof(a));
    a.dim = c->dim;
    a.ld = c->ld ? c->ld : ((c->dim + 31u) & ~31u);
    a.window = c->window_mode ? (c->window + 1u) / 2u : c->window;
    a.negatives = c->negatives;
    *floats_per_wave = w2v::train_snap_floats(a);
    return (uint64_t)*floats_per_wave * 4u * w2v::kMaxSummedWaves;
}

float *workspace_snap(const w2v_ctx *ctx)
{
    return reinterpret_cast<float *>(static_cast<unsigned char *>(ctx->cfg.workspace) + ctx->ws.snap_off);
}

// Queues one launch of the window kernel over the sentences described by `a`: picks the update mode and the
// number of wavefronts, plans the units on the device, launches.
// snap / snap_waves: where the summed mode keeps its snapshots and for how many wavefronts there is room.
int queue_launch(w2v_ctx *ctx, w2v::KernelArgs &a, float *snap, uint64_t snap_waves)
{
    const w2v_config &c = ctx->cfg;
    // Summed updates when wavefronts run side by side and either the caller asks for them or (automatic) the
    // counts say that the corpus spreads its tokens over far more rows than an L2 holds.
    int update = (c.update_mode == 2u || (c.update_mode == 0u && ctx->flat_corpus)) && ctx->snap_floats ? 1 : 0;
    if (c.sentences_in_flight == 1u) update = 0;       // strict order: nothing to sum
    if (ctx->forced_update >= 0) update = ctx->forced_update;
    if (c.storage) update = 2;                         // bfloat16 tables: their own kernels, always overwriting
    uint64_t waves = c.sentences_in_flight;
    if (waves == 0) {
        if (ctx->resident_waves[update] == 0) ctx->resident_waves[update] = w2v::train_resident_waves(a, update, c.device);
        waves = ctx->resident_waves[update];
        if (waves == 0) return fail(ctx, W2V_EHIP, "could not query kernel occupancy");
        waves = lock_free_waves(ctx, waves, update);
    }
    if (update == 1) {
        if (c.sentences_in_flight > snap_waves)
            return fail(ctx, W2V_EINVAL, "cfg.sentences_in_flight: the scratch memory holds the ring snapshots of " +
                                             std::to_string(snap_waves) + " wavefronts with summed updates (" +
                                             std::to_string((uint64_t)ctx->snap_floats * 4u) + " bytes each)");
        if (waves > snap_waves) waves = snap_waves;
        a.snap = snap;
        a.snap_stride = ctx->snap_floats;
    }
    if (a.n_sent < 65536u && waves > (a.n_sent << 16)) waves = a.n_sent << 16;   // a sentence is never cut into more units than that
    w2v::PlanRequest rq;
    rq.n_sent = a.n_sent;
    rq.waves = waves;
    rq.forced_unit_shift = ctx->forced_unit_shift;
    rq.forced_fine_shift = ctx->forced_fine_shift;
    rq.forced_coarse_sent = ctx->forced_coarse_sent;
    HIP_TRY(ctx, w2v::launch_plan(a.accum, a.sent_off, rq, stream_of(ctx)));
    HIP_TRY(ctx, w2v::launch_train(a, update, (uint32_t)waves, stream_of(ctx)));
    ctx->last_update = update;
    ctx->last_waves = waves;
    return W2V_OK;
}

}  // namespace

extern "C" {

int w2v_query_ld(uint32_t dim, uint32_t *ld_out)
{
    if (!ld_out || dim < 1 || dim > W2V_MAX_DIM) return W2V_EINVAL;
    *ld_out = (dim + 31u) & ~31u;     // 32 floats = one 128-byte line
    return W2V_OK;
}

int w2v_query_workspace(const w2v_config *cfg, uint32_t table_size, uint64_t *bytes_out)
{
    if (!cfg || !bytes_out || cfg->vocab < 1 || cfg->vocab > W2V_MAX_VOCAB || table_size < 1 || table_size > (1u << 31))
        return W2V_EINVAL;
    uint32_t per_wave = 0;
    uint64_t snap = 0;
    if (cfg->dim >= 1 && cfg->dim <= W2V_MAX_DIM && cfg->window >= 1 && cfg->window <= W2V_MAX_WINDOW &&
        cfg->negatives <= W2V_MAX_NEGATIVES && cfg->update_mode <= 2u)
        snap = snapshot_bytes(cfg, &per_wave);
    *bytes_out = w2v::workspace_layout(cfg->vocab, table_size, snap).total;
    return W2V_OK;
}

int w2v_create(const w2v_config *cfg, int init_weights, w2v_ctx **out)
{
    if (!out) return fail(nullptr, W2V_EINVAL, "out is NULL");
    *out = nullptr;
    const std::string why = check_config(cfg);
    if (!why.empty()) return fail(nullptr, W2V_EINVAL, why);
    uint32_t snap_floats = 0;
    const uint64_t snap_bytes = snapshot_bytes(cfg, &snap_floats);
    if (cfg->storage == 1u) {
        w2v::KernelArgs probe;
        std::memset(&probe, 0, sizeof(probe));
        probe.dim = cfg->dim;
        probe.ld = cfg->ld;
        probe.window = cfg->window_mode ? (cfg->window + 1u) / 2u : cfg->window;
        probe.negatives = cfg->negatives;
        if (!w2v::train_kernel_exists(probe, 2))
            return fail(nullptr, W2V_EINVAL, "cfg.storage 1 (bfloat16 tables) needs dim <= 320 in a 4-element layout (or <= 128 even, or <= 64), "
                                             "window <= 10 (as it occurs) and 5 to 11 negatives");
    }
    if (cfg->update_mode == 2u && snap_floats == 0)
        return fail(nullptr, W2V_EINVAL, "cfg.update_mode 2 (summed updates) needs dim <= 256, window <= 10 (as it occurs) and 5 to 11 negatives");
    const w2v::WorkspaceLayout minimal = w2v::workspace_layout(cfg->vocab, 1, snap_bytes);
    if (cfg->workspace_bytes < minimal.total) return fail(nullptr, W2V_ENOMEM, "cfg.workspace_bytes is smaller than w2v_query_workspace()");
    w2v_ctx *ctx = new (std::nothrow) w2v_ctx();
    if (!ctx) return fail(nullptr, W2V_ENOMEM, "out of host memory");
    ctx->cfg = *cfg;
    ctx->ws = minimal;
    ctx->snap_floats = snap_floats;
    hipError_t e = hipSetDevice(cfg->device);
    if (e == hipSuccess)
        e = w2v::launch_reset_accum(reinterpret_cast<w2v::Accum *>(static_cast<unsigned char *>(cfg->workspace)), 2, stream_of(ctx));
    if (e == hipSuccess && init_weights)
        e = w2v::launch_init_weights(cfg->syn0, cfg->syn1neg, cfg->vocab, cfg->dim, cfg->ld, cfg->seed, cfg->storage,
                                     stream_of(ctx));
    if (e != hipSuccess) {
        fail_hip(nullptr, e, "w2v_create");
        delete ctx;
        return W2V_EHIP;
    }
    *out = ctx;
    return W2V_OK;
}

int w2v_destroy(w2v_ctx *ctx)
{
    if (!ctx) return W2V_EINVAL;
    int rc = W2V_OK;
    if (hipSetDevice(ctx->cfg.device) != hipSuccess || hipStreamSynchronize(stream_of(ctx)) != hipSuccess) rc = W2V_EHIP;
    if (ctx->copy_stream) {
        if (hipStreamSynchronize(ctx->copy_stream) != hipSuccess) rc = W2V_EHIP;
        for (int h = 0; h < 2; ++h) {
            if (ctx->filled[h]) (void)hipEventDestroy(ctx->filled[h]);
            if (ctx->drained[h]) (void)hipEventDestroy(ctx->drained[h]);
        }
        (void)hipStreamDestroy(ctx->copy_stream);
    }
    delete ctx;
    return rc;
}

int w2v_build_unigram_table(w2v_ctx *ctx, const uint64_t *counts_host, uint32_t table_size)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    if (!counts_host) return fail(ctx, W2V_EINVAL, "counts_host is NULL");
    if (table_size < 1 || table_size > (1u << 31)) return fail(ctx, W2V_EINVAL, "table_size out of range [1, 2^31]");
    const uint32_t V = ctx->cfg.vocab;
    const w2v::WorkspaceLayout lay = w2v::workspace_layout(V, table_size, (uint64_t)ctx->snap_floats * 4u * w2v::kMaxSummedWaves);
    if (ctx->cfg.workspace_bytes < lay.total) return fail(ctx, W2V_ENOMEM, "workspace too small for this table_size");

    // share of word i: count_i^(3/4) = sqrt(c) * sqrt(sqrt(c)), accumulated in id order
    double total_w = 0.0, total_c = 0.0;
    for (uint32_t i = 0; i < V; ++i) {
        const double c = (double)counts_host[i];
        total_w += std::sqrt(c) * std::sqrt(std::sqrt(c));
        total_c += c;
    }
    if (!(total_w > 0.0)) return fail(ctx, W2V_EINVAL, "all counts are zero");

    std::vector<int32_t> table(table_size);
    {
        double cum = 0.0;
        uint64_t begin = 0;
        for (uint32_t i = 0; i < V; ++i) {
            const double c = (double)counts_host[i];
            cum += std::sqrt(c) * std::sqrt(std::sqrt(c));
            uint64_t end = (uint64_t)std::floor((cum / total_w) * (double)table_size);
            if (end > table_size || i == V - 1) end = table_size;
            for (uint64_t sl = begin; sl < end; ++sl) table[sl] = (int32_t)i;
            if (end > begin) begin = end;
        }
    }
    // keep probability min(1, sqrt(t / f)), f = count / total, as a 32-bit threshold
    std::vector<uint32_t> thr(V, 0xFFFFFFFFu);
    const double t = ctx->cfg.subsample_t;
    double kept_c = total_c;                       // expected count of the tokens that survive subsampling
    double kept_sq = 0.0;                          // ... and the sum of the squares of the words' expected kept counts
    for (uint32_t i = 0; i < V; ++i) {
        if (counts_host[i] == 0) continue;
        double keep = 1.0;
        if (t > 0.0) {
            const double f = (double)counts_host[i] / total_c;
            const double p = std::sqrt(t / f);
            if (p < 1.0) {
                const double q = std::floor(p * 4294967296.0);
                thr[i] = q >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)q;
                kept_c -= (1.0 - p) * (double)counts_host[i];
                keep = p;
            }
        }
        kept_sq += (keep * (double)counts_host[i]) * (keep * (double)counts_host[i]);
    }
    ctx->kept_fraction = kept_c / total_c;
    ctx->collision_mass = kept_c > 0.0 ? kept_sq / (kept_c * kept_c) : 0.0;
    // Share of the tokens carried by the rows that fit one XCD's L2 (2 MB of each table): small for walks over a
    // large graph, large for text.  Where it is small the frequent rows are not held in L2 anyway, and it is exactly
    // those rows whose copies must not diverge between XCDs: such corpora get summed, system-scope updates.
    {
        std::vector<uint64_t> by_count(counts_host, counts_host + V);
        const size_t rows = std::min<size_t>(V, std::max<size_t>(1, (2u << 20) / ((size_t)ctx->cfg.ld * 4u)));
        std::nth_element(by_count.begin(), by_count.begin() + (rows - 1), by_count.end(), std::greater<uint64_t>());
        double top = 0.0;
        for (size_t i = 0; i < rows; ++i) top += (double)by_count[i];
        ctx->flat_corpus = top < 0.30 * total_c;
    }

    unsigned char *ws = static_cast<unsigned char *>(ctx->cfg.workspace);
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    HIP_TRY(ctx, hipMemcpy(ws + lay.thr_off, thr.data(), (size_t)V * sizeof(uint32_t), hipMemcpyHostToDevice));
    HIP_TRY(ctx, hipMemcpy(ws + lay.table_off, table.data(), (size_t)table_size * sizeof(int32_t), hipMemcpyHostToDevice));
    ctx->ws = lay;
    ctx->table_size = table_size;
    ctx->table_built = true;
    return W2V_OK;
}

int w2v_train_epoch(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev, uint64_t n_sent,
                    uint64_t first_token_global_pos, uint32_t epoch)
{
    const int rc = check_train_call(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    if (rc != W2V_OK) return rc;
    if (n_sent == 0) return W2V_OK;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    w2v::KernelArgs a = kernel_args(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    return queue_launch(ctx, a, workspace_snap(ctx), w2v::kMaxSummedWaves);
}

int w2v_train_epoch_static(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev, uint64_t n_sent,
                           uint64_t first_token_global_pos, uint32_t epoch, double *loss_sum_dev, uint64_t *pairs_dev)
{
    const int rc = check_train_call(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    if (rc != W2V_OK) return rc;
    // the scratch array: accumulator block first, then the snapshot rows of as many wavefronts as fit
    const uint64_t head = 256;
    const uint64_t per_wave = (uint64_t)ctx->snap_floats * 4u;
    const uint64_t snap_waves = per_wave ? (w2v::kStaticScratchBytes - head) / per_wave : 0;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    unsigned char *scratch = nullptr;
    HIP_TRY(ctx, w2v::static_scratch(ctx->cfg.device, &scratch));
    w2v::KernelArgs a = kernel_args(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    a.accum = reinterpret_cast<w2v::Accum *>(scratch);
    // the array keeps what the last call left: the accumulators start from zero (a kernel, not a memset, so that the
    // call may be captured into a graph); the snapshot rows are written before they are read
    HIP_TRY(ctx, w2v::launch_reset_accum(a.accum, 2, stream_of(ctx)));
    if (n_sent) {
        const int qrc = queue_launch(ctx, a, reinterpret_cast<float *>(scratch + head), snap_waves);
        if (qrc != W2V_OK) return qrc;
    }
    HIP_TRY(ctx, w2v::launch_export_accum(a.accum, loss_sum_dev, pairs_dev, stream_of(ctx)));
    return W2V_OK;
}

int w2v_train_epoch_host(w2v_ctx *ctx, const int32_t *tokens_host, const uint64_t *sent_off_host, uint64_t n_sent,
                         uint64_t first_token_global_pos, uint32_t epoch, void *staging_dev, uint64_t staging_bytes)
{
    const int rc = check_train_call(ctx, tokens_host, sent_off_host, n_sent, first_token_global_pos, epoch);
    if (rc != W2V_OK) return rc;
    if (!staging_dev || ((uintptr_t)staging_dev & 255u) != 0)
        return fail(ctx, W2V_EINVAL, "staging_dev is NULL or not 256-byte aligned");
    const uint64_t half = (staging_bytes / 2u) & ~(uint64_t)255u;
    // a batch of n tokens in k sentences takes 4n bytes of ids, padding to 8, and 8(k+1) bytes of offsets
    auto batch_bytes = [](uint64_t ntok, uint64_t nsent) { return ((4u * ntok + 7u) & ~(uint64_t)7u) + 8u * (nsent + 1u); };
    for (uint64_t s = 0; s < n_sent; ++s) {
        if (sent_off_host[s + 1] < sent_off_host[s]) return fail(ctx, W2V_EINVAL, "sent_off_host is not non-decreasing");
        if (batch_bytes(sent_off_host[s + 1] - sent_off_host[s], 1) > half)
            return fail(ctx, W2V_EINVAL, "a sentence does not fit half of the staging buffer");
    }
    if (n_sent == 0) return W2V_OK;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    if (!ctx->copy_stream) {
        HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->copy_stream, hipStreamNonBlocking));
        for (int h = 0; h < 2; ++h) {
            HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->filled[h], hipEventDisableTiming));
            HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->drained[h], hipEventDisableTiming | hipEventBlockingSync));
        }
    }
    // Batches of nearly equal size, as few as fit: a full half followed by a small rest would leave the small
    // batch's launch as the only cover for the next large copy.
    const uint64_t all_bytes = batch_bytes(sent_off_host[n_sent] - sent_off_host[0], n_sent);
    const uint64_t n_batches = (all_bytes + half - 1u) / half;
    const uint64_t goal = (all_bytes + n_batches - 1u) / n_batches;          // bytes per batch aimed at (<= half)
    uint64_t s0 = 0;
    while (s0 < n_sent) {
        uint64_t s1 = s0 + 1;
        while (s1 < n_sent && batch_bytes(sent_off_host[s1] - sent_off_host[s0], s1 - s0) < goal &&
               batch_bytes(sent_off_host[s1 + 1] - sent_off_host[s0], s1 + 1 - s0) <= half) ++s1;
        // the halves alternate from batch to batch, across calls as well: the first batch of an epoch is copied
        // while the last batch of the epoch before it still trains
        const int h = ctx->next_half;
        ctx->next_half ^= 1;
        const uint64_t t_begin = sent_off_host[s0], ntok = sent_off_host[s1] - t_begin, nsent = s1 - s0;
        unsigned char *base = static_cast<unsigned char *>(staging_dev) + (uint64_t)h * half;
        int32_t *tok_dev = reinterpret_cast<int32_t *>(base);
        uint64_t *off_dev = reinterpret_cast<uint64_t *>(base + ((4u * ntok + 7u) & ~(uint64_t)7u));
        // Refill this half only after the batch that used it last (two steps ago, or in an earlier call) has
        // been trained.  The host waits for that too, so it is never more than two batches ahead of the GPU:
        // with hundreds of copies and launches queued ahead the runtime's own throttle sets in, copies then
        // block for a whole epoch at a time and the pipeline runs dry (measured: 20 ms per epoch instead of 10.5).
        if (ctx->drained_recorded[h]) {
            HIP_TRY(ctx, hipEventSynchronize(ctx->drained[h]));
            HIP_TRY(ctx, hipStreamWaitEvent(ctx->copy_stream, ctx->drained[h], 0));
        }
        if (ntok) HIP_TRY(ctx, hipMemcpyAsync(tok_dev, tokens_host + t_begin, 4u * ntok, hipMemcpyHostToDevice, ctx->copy_stream));
        HIP_TRY(ctx, hipMemcpyAsync(off_dev, sent_off_host + s0, 8u * (nsent + 1u), hipMemcpyHostToDevice, ctx->copy_stream));
        HIP_TRY(ctx, hipEventRecord(ctx->filled[h], ctx->copy_stream));
        HIP_TRY(ctx, hipStreamWaitEvent(stream_of(ctx), ctx->filled[h], 0));
        // The offsets keep their values from the whole corpus; the token pointer is moved back by the
        // batch's first offset instead, so positions (random keys, learning rate) are those of the corpus.
        const int32_t *tok_moved = reinterpret_cast<const int32_t *>(reinterpret_cast<uintptr_t>(tok_dev) - 4u * t_begin);
        w2v::KernelArgs a = kernel_args(ctx, tok_moved, off_dev, nsent, first_token_global_pos, epoch);
        const int qrc = queue_launch(ctx, a, workspace_snap(ctx), w2v::kMaxSummedWaves);
        if (qrc != W2V_OK) return qrc;
        HIP_TRY(ctx, hipEventRecord(ctx->drained[h], stream_of(ctx)));
        ctx->drained_recorded[h] = true;
        s0 = s1;
    }
    return W2V_OK;
}

int w2v_train_epoch_naive(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev, uint64_t n_sent,
                          uint64_t first_token_global_pos, uint32_t epoch)
{
    const int rc = check_train_call(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    if (rc != W2V_OK) return rc;
    if (ctx->cfg.negative_block > 1u)
        return fail(ctx, W2V_EINVAL, "the no-reuse comparator draws fresh negatives per window (cfg.negative_block must be 0 or 1)");
    if (ctx->cfg.storage) return fail(ctx, W2V_EINVAL, "the no-reuse comparator works on float tables (cfg.storage must be 0)");
    if (n_sent == 0) return W2V_OK;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    const w2v::KernelArgs a = kernel_args(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    uint64_t waves = ctx->cfg.sentences_in_flight;
    if (waves == 0) {
        waves = w2v::naive_resident_waves(ctx->cfg.device);
        if (waves == 0) return fail(ctx, W2V_EHIP, "could not query kernel occupancy");
    }
    if (waves > n_sent) waves = n_sent;
    HIP_TRY(ctx, w2v::launch_reset_accum(a.accum, 1, stream_of(ctx)));
    HIP_TRY(ctx, w2v::launch_train_naive(a, (uint32_t)waves, stream_of(ctx)));
    return W2V_OK;
}

int w2v_get_embeddings(w2v_ctx *ctx, int which, float *dst, uint64_t dst_floats, int dst_is_device)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    if (which != 0 && which != 1) return fail(ctx, W2V_EINVAL, "which must be 0 (syn0) or 1 (syn1neg)");
    if (!dst) return fail(ctx, W2V_EINVAL, "dst is NULL");
    const w2v_config &c = ctx->cfg;
    if (dst_floats < (uint64_t)c.vocab * c.dim) return fail(ctx, W2V_EINVAL, "dst_floats is smaller than vocab*dim");
    HIP_TRY(ctx, hipSetDevice(c.device));
    const void *src = which == 0 ? c.syn0 : c.syn1neg;
    if (c.storage) {
        if (!dst_is_device)
            return fail(ctx, W2V_EINVAL, "bfloat16 tables are widened on the device: dst must be device memory (dst_is_device != 0)");
        HIP_TRY(ctx, w2v::launch_widen_rows(src, dst, c.vocab, c.dim, c.ld, stream_of(ctx)));
        HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
        return W2V_OK;
    }
    HIP_TRY(ctx, hipMemcpy2DAsync(dst, (size_t)c.dim * sizeof(float), src, (size_t)c.ld * sizeof(float),
                                  (size_t)c.dim * sizeof(float), c.vocab,
                                  dst_is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, stream_of(ctx)));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    return W2V_OK;
}

int w2v_loss(w2v_ctx *ctx, double *loss_sum, uint64_t *positive_pairs, int reset)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    w2v::Accum host;
    w2v::Accum *dev = reinterpret_cast<w2v::Accum *>(static_cast<unsigned char *>(ctx->cfg.workspace) + ctx->ws.accum_off);
    HIP_TRY(ctx, hipMemcpyAsync(&host, dev, sizeof(host), hipMemcpyDeviceToHost, stream_of(ctx)));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    if (loss_sum) *loss_sum = host.loss_sum;
    if (positive_pairs) *positive_pairs = host.pairs;
    if (reset) HIP_TRY(ctx, w2v::launch_reset_accum(dev, 2, stream_of(ctx)));
    return W2V_OK;
}

int w2v_counters(w2v_ctx *ctx, uint64_t *kept_tokens, uint64_t *invalid_tokens, int reset)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    w2v::Accum host;
    w2v::Accum *dev = reinterpret_cast<w2v::Accum *>(static_cast<unsigned char *>(ctx->cfg.workspace) + ctx->ws.accum_off);
    HIP_TRY(ctx, hipMemcpyAsync(&host, dev, sizeof(host), hipMemcpyDeviceToHost, stream_of(ctx)));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    if (kept_tokens) *kept_tokens = host.kept;
    if (invalid_tokens) *invalid_tokens = host.dropped;
    if (reset) HIP_TRY(ctx, w2v::launch_reset_accum(dev, 2, stream_of(ctx)));
    return W2V_OK;
}

int w2v_debug_draws(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev, uint64_t n_sent,
                    uint64_t first_token_global_pos, uint32_t epoch, uint8_t *keep_dev, uint8_t *width_dev,
                    int32_t *neg_dev)
{
    const int rc = check_train_call(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    if (rc != W2V_OK) return rc;
    if (!keep_dev || !width_dev || (ctx->cfg.negatives && !neg_dev)) return fail(ctx, W2V_EINVAL, "an output pointer is NULL");
    if (n_sent == 0) return W2V_OK;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    uint64_t n_tokens = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&n_tokens, sent_off_dev + n_sent, sizeof(uint64_t), hipMemcpyDeviceToHost, stream_of(ctx)));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    const w2v::KernelArgs a = kernel_args(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    HIP_TRY(ctx, w2v::launch_draws(a, n_tokens, keep_dev, width_dev, neg_dev, stream_of(ctx)));
    return W2V_OK;
}

int w2v_debug_train_draws(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev, uint64_t n_sent,
                          uint64_t first_token_global_pos, uint32_t epoch, uint8_t *keep_dev, uint8_t *width_dev,
                          int32_t *neg_dev)
{
    const int rc = check_train_call(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    if (rc != W2V_OK) return rc;
    if (!keep_dev || !width_dev || (ctx->cfg.negatives && !neg_dev)) return fail(ctx, W2V_EINVAL, "an output pointer is NULL");
    if (n_sent == 0) return W2V_OK;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    uint64_t n_tokens = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&n_tokens, sent_off_dev + n_sent, sizeof(uint64_t), hipMemcpyDeviceToHost, stream_of(ctx)));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    w2v::KernelArgs a = kernel_args(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch);
    a.dump.keep = keep_dev;
    a.dump.width = width_dev;
    a.dump.neg = neg_dev;
    HIP_TRY(ctx, w2v::launch_fill_dump(a.dump, n_tokens, ctx->cfg.negatives, stream_of(ctx)));
    return queue_launch(ctx, a, workspace_snap(ctx), w2v::kMaxSummedWaves);
}

int w2v_debug_set_update(w2v_ctx *ctx, int update)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    if (update < -1 || update > 1) return fail(ctx, W2V_EINVAL, "update must be -1 (by the rules), 0 (overwrite) or 1 (summed)");
    if (update == 1 && ctx->snap_floats == 0) return fail(ctx, W2V_EINVAL, "no summed-update kernel for this configuration");
    ctx->forced_update = update;
    return W2V_OK;
}

int w2v_debug_get_plan(w2v_ctx *ctx, uint32_t *unit_shift, uint32_t *fine_shift, uint64_t *coarse_sentences, uint64_t *units,
                       uint32_t *update, uint64_t *wavefronts)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    w2v::Accum host;
    w2v::Accum *dev = reinterpret_cast<w2v::Accum *>(static_cast<unsigned char *>(ctx->cfg.workspace) + ctx->ws.accum_off);
    HIP_TRY(ctx, hipMemcpyAsync(&host, dev, sizeof(host), hipMemcpyDeviceToHost, stream_of(ctx)));
    HIP_TRY(ctx, hipStreamSynchronize(stream_of(ctx)));
    if (unit_shift) *unit_shift = host.unit_shift;
    if (fine_shift) *fine_shift = host.fine_shift;
    if (coarse_sentences) *coarse_sentences = host.coarse_sent;
    if (units) *units = host.n_units;
    if (update) *update = (uint32_t)ctx->last_update;
    if (wavefronts) *wavefronts = ctx->last_waves;
    return W2V_OK;
}

int w2v_debug_set_units(w2v_ctx *ctx, int unit_shift)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    if (unit_shift < -1 || unit_shift > 16) return fail(ctx, W2V_EINVAL, "unit_shift must be -1 (automatic) or 0..16");
    ctx->forced_unit_shift = unit_shift;
    return W2V_OK;
}

int w2v_debug_set_unit_tail(w2v_ctx *ctx, int fine_shift, uint64_t coarse_sentences)
{
    if (!ctx) return fail(nullptr, W2V_EINVAL, "ctx is NULL");
    if (fine_shift < -1 || fine_shift > 16) return fail(ctx, W2V_EINVAL, "fine_shift must be -1 (automatic) or 0..16");
    ctx->forced_fine_shift = fine_shift;
    ctx->forced_coarse_sent = coarse_sentences;
    return W2V_OK;
}

int w2v_debug_reduce(const float *in_dev, float *out_dev, void *stream)
{
    if (!in_dev || !out_dev) return W2V_EINVAL;
    return w2v::launch_reduce_selftest(in_dev, out_dev, static_cast<hipStream_t>(stream)) == hipSuccess ? W2V_OK : W2V_EHIP;
}

const char *w2v_last_error(const w2v_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
