// Host side of the DEF / DEF-A step library: the C ABI declared in include/def.h.
// Validation, the shared block draw, state allocation and kernel sequencing.
// No arithmetic of the method happens on the host except the O(1) block draw
// (arXiv 2004.05298, Sec. 1: one uniformly sampled start index per iteration).
#include "def.h"
#include "def_internal.h"

#include <cstring>
#include <new>
#include <vector>

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t err)
{
    g_last_hip_error = (int)err;
    (void)hipGetLastError();   // clear the sticky error so that later calls start clean
    return err == hipErrorOutOfMemory ? DEF_ENOMEM : DEF_EHIP;
}

#define DEF_HIP(call)                                   \
    do {                                                \
        hipError_t err__ = (call);                      \
        if (err__ != hipSuccess) return hip_fail(err__); \
    } while (0)

// Philox4x64-10 (Salmon, Moraes, Dror, Shaw, SC 2011): ten rounds of two
// 64x64->128-bit multiplications whose halves are crossed with the other counter
// words and the key; the key advances by the Weyl constants between rounds.
void philox4x64_10(uint64_t ctr[4], const uint64_t key_in[2])
{
    const uint64_t mul0 = 0xD2E7470EE14C6C93ull, mul1 = 0xCA5A826395121157ull;
    const uint64_t weyl0 = 0x9E3779B97F4A7C15ull, weyl1 = 0xBB67AE8584CAA73Bull;
    uint64_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        const unsigned __int128 p0 = (unsigned __int128)mul0 * ctr[0];
        const unsigned __int128 p1 = (unsigned __int128)mul1 * ctr[2];
        const uint64_t n0 = (uint64_t)(p1 >> 64) ^ ctr[1] ^ k0;
        const uint64_t n1 = (uint64_t)p1;
        const uint64_t n2 = (uint64_t)(p0 >> 64) ^ ctr[3] ^ k1;
        const uint64_t n3 = (uint64_t)p0;
        ctr[0] = n0; ctr[1] = n1; ctr[2] = n2; ctr[3] = n3;
        k0 += weyl0;
        k1 += weyl1;
    }
}

uint64_t draw_start(uint64_t seed, uint64_t t, uint64_t d)
{
    uint64_t ctr[4] = {t, 0, 0, 0};
    const uint64_t key[2] = {seed, 0};
    philox4x64_10(ctr, key);
    return ctr[0] % d;
}

uint64_t round_up(uint64_t v, uint64_t to) { return (v + to - 1) / to * to; }

// Makes one GPU current for the duration of a call and puts the caller's back afterwards.
class DeviceScope {
public:
    explicit DeviceScope(int device)
    {
        err_ = hipGetDevice(&prev_);
        if (err_ == hipSuccess && prev_ != device) {
            err_ = hipSetDevice(device);
            switched_ = err_ == hipSuccess;
        }
    }
    ~DeviceScope()
    {
        if (switched_) (void)hipSetDevice(prev_);
    }
    DeviceScope(const DeviceScope &) = delete;
    DeviceScope &operator=(const DeviceScope &) = delete;
    hipError_t status() const { return err_; }

private:
    int prev_ = -1;
    bool switched_ = false;
    hipError_t err_ = hipSuccess;
};

// Every entry point that reaches the HIP runtime runs on the GPU the context was made on.
#define DEF_ON_DEVICE(c)                                              \
    DeviceScope scope__((c)->device);                                 \
    if (scope__.status() != hipSuccess) return hip_fail(scope__.status())

}  // namespace

struct def_ctx {
    // problem
    uint64_t d = 0, B = 0, seed = 0, t = 0;
    uint32_t W = 0, R = 0, L = 0;
    float lr = 0, mu = 0, wd = 0;
    int64_t forced = -1;
    uint64_t last_start = 0;
    bool has_last = false;
    int last_flat = 0;
    bool pending_apply = false;   // def_pack has run, def_apply has not
    hipStream_t stream = nullptr;
    int device = 0;           // GPU that was current in def_init; owns the stream and all buffers
    // device state owned by the library
    float *e = nullptr, *m = nullptr, *msg = nullptr, *avg = nullptr;
    void *e_alloc = nullptr, *m_alloc = nullptr;   // what hipMalloc returned (e and m point inside)
    double *diag = nullptr;   // per-workgroup partial sums of def_diagnostics
    double *diag_workers = nullptr;   // per-workgroup partial sums of def_diagnostics_workers
    DefCtl *ctl = nullptr;    // device copy of (t, seed, forced, s) for the device draw
    bool device_draw = false;
    uint64_t ld = 0, ldmsg = 0;
    uint64_t *d_off = nullptr;
    uint32_t *d_tile_tensor = nullptr;   // tensor holding the first index of each tile
    // parameters
    float *x_flat = nullptr;
    float **d_xptrs = nullptr;
    // detached evaluation points requested with def_set_detach
    float *w = nullptr;
    uint64_t ldw = 0;
    float lam = 0;
    // gradient pointer table (tensor mode)
    // a few recently used tables are kept on the device, so that a caller cycling
    // through a handful of gradient sets pays for each upload once
    struct GradTable {
        std::vector<const float *> host;
        const float **dev = nullptr;
        uint64_t last_used = 0;
        bool captured = false;        // a captured graph reads this table: never replaced
    };
    std::vector<GradTable> gtab;
    uint64_t gtab_clock = 0;
    // per-launch timing of the streaming kernel
    std::vector<hipEvent_t> ev;
    uint32_t prof_cap = 0, prof_n = 0;
    char kernel_name[160] = {0};
};

namespace {

void free_ctx(def_ctx *c)
{
    if (!c) return;
    for (hipEvent_t ev : c->ev) (void)hipEventDestroy(ev);
    (void)hipFree(c->e_alloc);
    (void)hipFree(c->m_alloc);
    (void)hipFree(c->msg);
    (void)hipFree(c->avg);
    (void)hipFree(c->diag);
    (void)hipFree(c->diag_workers);
    (void)hipFree(c->ctl);
    (void)hipFree(c->d_off);
    (void)hipFree(c->d_tile_tensor);
    (void)hipFree(c->d_xptrs);
    for (auto &tb : c->gtab) (void)hipFree(tb.dev);
    delete c;
}

DefStepArgs base_args(const def_ctx *c, uint64_t s)
{
    DefStepArgs a{};
    a.d = c->d; a.B = c->B; a.s = s; a.W = c->W;
    a.backwards = (uint32_t)(c->t & 1u);
    a.lr = c->lr; a.mu = c->mu; a.wd = c->wd;
    a.e = c->e; a.m = c->m; a.ld = c->ld;
    a.msg = c->msg; a.ldmsg = c->ldmsg; a.avg = c->avg;
    a.x_flat = c->x_flat; a.x_ptrs = c->d_xptrs; a.off = c->d_off; a.L = c->L;
    a.tile_tensor = c->d_tile_tensor;
    a.w = c->w; a.ldw = c->ldw; a.lam = c->lam;
    return a;
}

// The part of an iteration that is local to the workers: block draw and streaming pass.
int run_stream(def_ctx *c, DefStepArgs &a)
{
    if (c->device_draw) {
        // the kernels take the start the draw kernel leaves in device memory; a.s, drawn
        // on the host from the host's copy of (seed, t), is the same number as long as
        // the host's step counter is current (see def_sync_step)
        DEF_HIP(def_launch_draw(c->ctl, c->d, c->stream));
        a.ctl = c->ctl;
    }
    const bool prof = c->prof_n < c->prof_cap;
    if (prof) DEF_HIP(hipEventRecord(c->ev[2 * c->prof_n], c->stream));
    {
        const hipError_t err = def_launch_stream(a, c->stream);
        if (err != hipSuccess) {
            // the draw kernel is already enqueued and will advance the device's step counter;
            // put the device copy back to the host's (t, forced start), which have not moved
            if (c->device_draw)
                (void)def_launch_ctl_set(c->ctl, DEF_CTL_T | DEF_CTL_FORCED, c->t, 0, c->forced, c->stream);
            return hip_fail(err);
        }
    }
    if (prof) {
        DEF_HIP(hipEventRecord(c->ev[2 * c->prof_n + 1], c->stream));
        ++c->prof_n;
    }
    c->last_start = a.s;
    c->has_last = true;
    // 1: flat addressing; 0: gradients and/or the parameters the pass reads come through tables
    c->last_flat = (a.g_ptrs || ((a.wd != 0.0f || a.w) && a.x_ptrs)) ? 0 : 1;
    def_describe_stream_kernel(a, c->kernel_name, sizeof c->kernel_name);
    c->forced = -1;
    ++c->t;
    return DEF_OK;
}

// The sequence of one iteration: streaming pass, average + update, optional y.
int run_step(def_ctx *c, DefStepArgs &a, float *y_out)
{
    const int rc = run_stream(c, a);
    if (rc != DEF_OK) return rc;
    DEF_HIP(def_launch_average_update(a, c->stream));
    if (y_out) DEF_HIP(def_launch_output(a, y_out, c->stream));
    return DEF_OK;
}

// First half of a split iteration: streaming pass, then the sum of the local workers' blocks.
int run_pack(def_ctx *c, DefStepArgs &a, const float **block_sum)
{
    const int rc = run_stream(c, a);
    if (rc != DEF_OK) return rc;
    DEF_HIP(def_launch_block_sum(a, c->stream));
    c->pending_apply = true;
    if (block_sum) *block_sum = c->avg;
    return DEF_OK;
}

uint64_t next_start(const def_ctx *c)
{
    return c->forced >= 0 ? (uint64_t)c->forced : draw_start(c->seed, c->t, c->d);
}

// The device copy of a table of W*L gradient pointers: one of the cached tables if the same
// pointers were seen recently, else uploaded into a free or the least recently used slot.
// While the stream is being captured nothing may be copied, and what the captured launch
// reads must stay as it is for every replay: a table that is not on the device yet is
// refused, and one that was used under capture is never replaced afterwards.
int device_grad_table(def_ctx *ctx, const float *const *grad_ptrs, const float ***out)
{
    const size_t n = (size_t)ctx->W * ctx->L;
    for (size_t q = 0; q < n; ++q)
        if (!grad_ptrs[q] || (uintptr_t)grad_ptrs[q] % 4 != 0) return DEF_EINVAL;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    DEF_HIP(hipStreamIsCapturing(ctx->stream, &capture));
    const bool capturing = capture != hipStreamCaptureStatusNone;
    def_ctx::GradTable *use = nullptr, *oldest = nullptr;
    size_t replaceable = 0;
    for (auto &tb : ctx->gtab) {
        if (tb.host.size() == n && std::memcmp(tb.host.data(), grad_ptrs, n * sizeof(float *)) == 0) {
            use = &tb;
            break;
        }
        if (!tb.captured) {
            ++replaceable;
            if (!oldest || tb.last_used < oldest->last_used) oldest = &tb;
        }
    }
    if (!use) {
        if (capturing) return DEF_EINVAL;      // run one eager step with this table first
        def_ctx::GradTable *slot = nullptr;
        if (replaceable >= DEF_GRAD_TABLES) {
            slot = oldest;
            // a step in flight may still read the table that is being replaced
            DEF_HIP(hipStreamSynchronize(ctx->stream));
        } else {
            try {
                ctx->gtab.emplace_back();
            } catch (const std::bad_alloc &) {
                return DEF_ENOMEM;
            }
            slot = &ctx->gtab.back();
            const hipError_t err = hipMalloc((void **)&slot->dev, n * sizeof(float *));
            if (err != hipSuccess) {
                ctx->gtab.pop_back();
                return hip_fail(err);
            }
        }
        slot->host.clear();                    // not a valid match until the copy has succeeded
        DEF_HIP(hipMemcpy(slot->dev, grad_ptrs, n * sizeof(float *), hipMemcpyHostToDevice));
        try {
            slot->host.assign(grad_ptrs, grad_ptrs + n);
        } catch (const std::bad_alloc &) {
            return DEF_ENOMEM;
        }
        use = slot;
    }
    use->last_used = ++ctx->gtab_clock;
    if (capturing) use->captured = true;
    *out = use->dev;
    return DEF_OK;
}

}  // namespace

extern "C" {

int def_block_start(uint64_t seed, uint64_t t, uint64_t d, uint64_t *start)
{
    if (!start || d == 0) return DEF_EINVAL;
    *start = draw_start(seed, t, d);
    return DEF_OK;
}

int def_init(def_ctx **out, const def_config *cfg)
{
    if (!out || !cfg) return DEF_EINVAL;
    if (cfg->d == 0 || cfg->d >= (1ull << 40) || cfg->W == 0 || cfg->R == 0 || cfg->R > cfg->d)
        return DEF_EINVAL;
    if (!(cfg->lr == cfg->lr) || !(cfg->momentum == cfg->momentum) ||
        !(cfg->weight_decay == cfg->weight_decay))
        return DEF_EINVAL;   // NaN hyper-parameters
    const uint32_t L = cfg->tensor_offsets ? cfg->n_tensors : 1;
    if (L == 0) return DEF_EINVAL;
    if (cfg->tensor_offsets) {
        if (cfg->tensor_offsets[0] != 0 || cfg->tensor_offsets[L] != cfg->d) return DEF_EINVAL;
        for (uint32_t l = 0; l < L; ++l)
            if (cfg->tensor_offsets[l] >= cfg->tensor_offsets[l + 1]) return DEF_EINVAL;
    }
    if (!cfg->params) {
        if (!cfg->param_ptrs) return DEF_EINVAL;
        for (uint32_t l = 0; l < L; ++l)
            if (!cfg->param_ptrs[l] || (uintptr_t)cfg->param_ptrs[l] % 4 != 0) return DEF_EINVAL;
    } else if ((uintptr_t)cfg->params % 4 != 0) {
        return DEF_EINVAL;
    }

    {
        // one workgroup per (worker, tile), up to 7 idle ones per worker: the grid must fit 31 bits
        const uint64_t grid_limit = 0x7fffffffull - 8;
        const uint64_t vec_tiles = (cfg->d + DEF_VEC_TILE - 1) / DEF_VEC_TILE;
        if ((vec_tiles + 7) * cfg->W > grid_limit) return DEF_EINVAL;
    }

    def_ctx *c = new (std::nothrow) def_ctx;
    if (!c) return DEF_ENOMEM;
    c->d = cfg->d; c->W = cfg->W; c->R = cfg->R; c->L = L;
    c->B = (cfg->d + cfg->R - 1) / cfg->R;                       // B = ceil(d/R)
    c->lr = cfg->lr; c->mu = cfg->momentum; c->wd = cfg->weight_decay;
    c->seed = cfg->seed;
    c->stream = (hipStream_t)cfg->stream;
    {
        const hipError_t err = hipGetDevice(&c->device);
        if (err != hipSuccess) { delete c; return hip_fail(err); }
    }
    c->x_flat = cfg->params;
    c->ld = round_up(c->d, DEF_STATE_ROW_MULTIPLE);
    c->ldmsg = round_up(c->B, DEF_AVG_TILE);

#define DEF_INIT_HIP(call)                                                      \
    do {                                                                        \
        hipError_t err__ = (call);                                              \
        if (err__ != hipSuccess) { free_ctx(c); return hip_fail(err__); }       \
    } while (0)

    const size_t state_bytes = (size_t)c->W * c->ld * sizeof(float);
    const size_t msg_bytes = (size_t)c->W * c->ldmsg * sizeof(float);
    // e and m start at fixed offsets past a multiple of DEF_STATE_SKEW_PERIOD bytes (see
    // def_internal.h: where the buffers sit relative to each other decides several points of bandwidth)
    DEF_INIT_HIP(hipMalloc(&c->e_alloc, state_bytes + DEF_STATE_SKEW_PERIOD + DEF_STATE_E_OFFSET));
    c->e = reinterpret_cast<float *>(round_up((uintptr_t)c->e_alloc, DEF_STATE_SKEW_PERIOD) + DEF_STATE_E_OFFSET);
    if (c->mu != 0.0f) {
        DEF_INIT_HIP(hipMalloc(&c->m_alloc, state_bytes + DEF_STATE_SKEW_PERIOD + DEF_STATE_M_OFFSET));
        c->m = reinterpret_cast<float *>(round_up((uintptr_t)c->m_alloc, DEF_STATE_SKEW_PERIOD) + DEF_STATE_M_OFFSET);
    }
    DEF_INIT_HIP(hipMalloc((void **)&c->msg, msg_bytes));
    DEF_INIT_HIP(hipMalloc((void **)&c->avg, c->ldmsg * sizeof(float)));
    DEF_INIT_HIP(hipMalloc((void **)&c->diag, def_diag_blocks(c->d) * 2 * sizeof(double)));
    DEF_INIT_HIP(hipMalloc((void **)&c->diag_workers,
                           def_diag_worker_blocks(c->d) * 2 * (size_t)c->W * sizeof(double)));
    DEF_INIT_HIP(hipMalloc((void **)&c->ctl, sizeof(DefCtl)));
    {
        // look the static scratch array of def_diagnostics_static up now, on this GPU, so that
        // a later call of it (possibly while the stream is being captured) finds it resolved
        double *unused = nullptr;
        DEF_INIT_HIP(def_static_scratch_address(&unused));
        def_prepare_diagnostics_workers();   // likewise: the grid of the per-worker statistics
    }
    DEF_INIT_HIP(hipMemsetAsync(c->ctl, 0, sizeof(DefCtl), c->stream));

    // (the large device buffers come first so that a problem that does not fit fails
    // before any host table is built)
    // host tables: offsets, and for every tile the tensor that holds its first index
    const uint64_t n_tiles = (c->d + DEF_VEC_TILE - 1) / DEF_VEC_TILE;
    std::vector<uint64_t> off(L + 1);
    std::vector<uint32_t> tile_tensor;
    try {
        if (cfg->tensor_offsets) off.assign(cfg->tensor_offsets, cfg->tensor_offsets + L + 1);
        else { off[0] = 0; off[1] = c->d; }
        tile_tensor.resize(n_tiles);
        uint32_t l = 0;
        for (uint64_t t = 0; t < n_tiles; ++t) {
            while (t * DEF_VEC_TILE >= off[l + 1]) ++l;
            tile_tensor[t] = l;
        }
    } catch (const std::bad_alloc &) {
        free_ctx(c);
        return DEF_ENOMEM;
    }
    DEF_INIT_HIP(hipMalloc((void **)&c->d_off, (L + 1) * sizeof(uint64_t)));
    DEF_INIT_HIP(hipMalloc((void **)&c->d_tile_tensor, n_tiles * sizeof(uint32_t)));
    DEF_INIT_HIP(hipMemsetAsync(c->e, 0, state_bytes, c->stream));           // e_{k,0} = 0
    if (c->m) DEF_INIT_HIP(hipMemsetAsync(c->m, 0, state_bytes, c->stream)); // m_{k,0} = 0
    DEF_INIT_HIP(hipMemsetAsync(c->msg, 0, msg_bytes, c->stream));
    DEF_INIT_HIP(hipMemsetAsync(c->avg, 0, c->ldmsg * sizeof(float), c->stream));
    DEF_INIT_HIP(hipMemcpyAsync(c->d_off, off.data(), (L + 1) * sizeof(uint64_t),
                                hipMemcpyHostToDevice, c->stream));
    DEF_INIT_HIP(hipMemcpyAsync(c->d_tile_tensor, tile_tensor.data(), n_tiles * sizeof(uint32_t),
                                hipMemcpyHostToDevice, c->stream));
    if (!c->x_flat) {
        DEF_INIT_HIP(hipMalloc((void **)&c->d_xptrs, L * sizeof(float *)));
        DEF_INIT_HIP(hipMemcpyAsync(c->d_xptrs, cfg->param_ptrs, L * sizeof(float *),
                                    hipMemcpyHostToDevice, c->stream));
    }
    DEF_INIT_HIP(hipStreamSynchronize(c->stream));   // host tables go out of scope below
#undef DEF_INIT_HIP
    *out = c;
    return DEF_OK;
}

int def_destroy(def_ctx *ctx)
{
    if (!ctx) return DEF_EINVAL;
    DeviceScope scope(ctx->device);
    hipError_t err = scope.status();
    if (err == hipSuccess) err = hipStreamSynchronize(ctx->stream);
    free_ctx(ctx);
    return err == hipSuccess ? DEF_OK : hip_fail(err);
}

int def_step(def_ctx *ctx, const float *grads, uint64_t ld, float *y_out)
{
    if (!ctx || !grads || ld < ctx->d || (uintptr_t)grads % 4 != 0 || ctx->pending_apply) return DEF_EINVAL;
    if (y_out && (uintptr_t)y_out % 4 != 0) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, next_start(ctx));
    a.g_flat = grads;
    a.ldg = ld;
    a.g_ptrs = nullptr;
    return run_step(ctx, a, y_out);
}

int def_pack(def_ctx *ctx, const float *grads, uint64_t ld, const float **block_sum)
{
    if (!ctx || !grads || ld < ctx->d || (uintptr_t)grads % 4 != 0 || ctx->pending_apply) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, next_start(ctx));
    a.g_flat = grads;
    a.ldg = ld;
    a.g_ptrs = nullptr;
    return run_pack(ctx, a, block_sum);
}

int def_pack_tensors(def_ctx *ctx, const float *const *grad_ptrs, const float **block_sum)
{
    if (!ctx || !grad_ptrs || ctx->pending_apply) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    const float **table = nullptr;
    const int rc = device_grad_table(ctx, grad_ptrs, &table);
    if (rc != DEF_OK) return rc;
    DefStepArgs a = base_args(ctx, next_start(ctx));
    a.g_flat = nullptr;
    a.ldg = 0;
    a.g_ptrs = table;
    return run_pack(ctx, a, block_sum);
}

int def_apply(def_ctx *ctx, const float *block, float divisor, float *y_out)
{
    if (!ctx || !block || (uintptr_t)block % 4 != 0 || !(divisor > 0.0f) || !ctx->pending_apply)
        return DEF_EINVAL;
    if (y_out && (uintptr_t)y_out % 4 != 0) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, ctx->last_start);
    if (ctx->device_draw) a.ctl = ctx->ctl;      // the start the pack half drew on the device
    DEF_HIP(def_launch_apply_block(a, block, divisor, ctx->stream));
    ctx->pending_apply = false;
    if (y_out) DEF_HIP(def_launch_output(a, y_out, ctx->stream));
    return DEF_OK;
}

int def_a_step(def_ctx *ctx, const float *grads, uint64_t ld)
{
    return def_step(ctx, grads, ld, nullptr);
}

int def_step_tensors(def_ctx *ctx, const float *const *grad_ptrs, float *y_out)
{
    if (!ctx || !grad_ptrs || ctx->pending_apply) return DEF_EINVAL;
    if (y_out && (uintptr_t)y_out % 4 != 0) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    const float **table = nullptr;
    const int rc = device_grad_table(ctx, grad_ptrs, &table);
    if (rc != DEF_OK) return rc;
    DefStepArgs a = base_args(ctx, next_start(ctx));
    a.g_flat = nullptr;
    a.ldg = 0;
    a.g_ptrs = table;
    return run_step(ctx, a, y_out);
}

int def_a_step_tensors(def_ctx *ctx, const float *const *grad_ptrs)
{
    return def_step_tensors(ctx, grad_ptrs, nullptr);
}

int def_output(def_ctx *ctx, float *y_out)
{
    if (!ctx || !y_out || (uintptr_t)y_out % 4 != 0) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, 0);
    DEF_HIP(def_launch_output(a, y_out, ctx->stream));
    return DEF_OK;
}

int def_set_detach(def_ctx *ctx, float *w_out, uint64_t ldw, float lambda)
{
    // between def_pack and def_apply the off-block points of the step in flight are already
    // written (or not): changing the destination there would leave them half done
    if (!ctx || ctx->pending_apply) return DEF_EINVAL;
    if (w_out) {
        if ((uintptr_t)w_out % 4 != 0 || ldw < ctx->d || !(lambda >= 0.0f && lambda <= 1.0f))
            return DEF_EINVAL;
        DEF_ON_DEVICE(ctx);
        // the points for the state as it is now (x_0 itself before the first step), so that
        // the buffer is valid from this call on and not only after the next step
        DefStepArgs a = base_args(ctx, 0);
        a.w = w_out; a.ldw = ldw; a.lam = lambda;
        DEF_HIP(def_launch_detach(a, ctx->stream));
        ctx->w = w_out; ctx->ldw = ldw; ctx->lam = lambda;
    } else {
        ctx->w = nullptr; ctx->ldw = 0; ctx->lam = 0.0f;
    }
    return DEF_OK;
}

int def_detach(def_ctx *ctx, float *w_out, uint64_t ldw, float lambda)
{
    if (!ctx || !w_out || (uintptr_t)w_out % 4 != 0 || ldw < ctx->d ||
        !(lambda >= 0.0f && lambda <= 1.0f))
        return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, 0);
    a.w = w_out; a.ldw = ldw; a.lam = lambda;
    DEF_HIP(def_launch_detach(a, ctx->stream));
    return DEF_OK;
}

int def_diagnostics(def_ctx *ctx, float lambda, double *out)
{
    if (!ctx || !out || (uintptr_t)out % 8 != 0 || !(lambda >= 0.0f && lambda <= 1.0f)) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, 0);
    DEF_HIP(def_launch_diagnostics(a, lambda, ctx->diag, out, ctx->stream));
    return DEF_OK;
}

int def_diagnostics_static(const float *e, uint64_t ld, uint64_t d, uint32_t W, float lambda, double *out,
                           void *stream)
{
    if (!e || !out || d == 0 || W == 0 || ld < d || ld % 4 != 0 || (uintptr_t)e % 16 != 0 ||
        (uintptr_t)out % 8 != 0 || !(lambda >= 0.0f && lambda <= 1.0f))
        return DEF_EINVAL;
    const uint64_t blocks = def_diag_blocks(d);
    if (blocks * 2 > DEF_STATIC_SCRATCH_DOUBLES) return DEF_ELIMIT;   // d > DEF_STATIC_MAX_D
    double *scratch = nullptr;
    DEF_HIP(def_static_scratch_address(&scratch));
    DefStepArgs a{};
    a.d = d; a.W = W; a.ld = ld;
    a.e = const_cast<float *>(e);                 // the statistics kernels only read it
    // every partial sum the second kernel reads is written by the first: nothing to clear
    DEF_HIP(def_launch_diagnostics(a, lambda, scratch, out, (hipStream_t)stream));
    return DEF_OK;
}

int def_diagnostics_workers(def_ctx *ctx, double *out)
{
    if (!ctx || !out || (uintptr_t)out % 8 != 0) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    DefStepArgs a = base_args(ctx, 0);
    DEF_HIP(def_launch_diagnostics_workers(a, ctx->diag_workers, out, ctx->stream));
    return DEF_OK;
}

int def_set_seed(def_ctx *ctx, uint64_t seed)
{
    if (!ctx) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    if (ctx->device_draw)
        DEF_HIP(def_launch_ctl_set(ctx->ctl, DEF_CTL_SEED, 0, seed, -1, ctx->stream));
    ctx->seed = seed;
    return DEF_OK;
}

int def_set_device_draw(def_ctx *ctx, int on)
{
    if (!ctx) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    if (on && !ctx->device_draw)
        DEF_HIP(def_launch_ctl_set(ctx->ctl, DEF_CTL_T | DEF_CTL_SEED | DEF_CTL_FORCED, ctx->t, ctx->seed,
                                   ctx->forced, ctx->stream));
    ctx->device_draw = on != 0;
    return DEF_OK;
}

int def_sync_step(def_ctx *ctx)
{
    if (!ctx) return DEF_EINVAL;
    if (!ctx->device_draw) return DEF_OK;
    DEF_ON_DEVICE(ctx);
    DefCtl host;
    DEF_HIP(hipMemcpyAsync(&host, ctx->ctl, sizeof host, hipMemcpyDeviceToHost, ctx->stream));
    DEF_HIP(hipStreamSynchronize(ctx->stream));
    if (host.t != ctx->t) {          // steps ran that the host did not issue itself (graph replays)
        ctx->last_start = host.s;
        ctx->has_last = host.t > 0;
    }
    ctx->t = host.t;
    ctx->forced = host.forced;
    return DEF_OK;
}

int def_set_lr(def_ctx *ctx, float lr)
{
    if (!ctx || !(lr == lr)) return DEF_EINVAL;
    ctx->lr = lr;
    return DEF_OK;
}

int def_set_step(def_ctx *ctx, uint64_t t)
{
    if (!ctx) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    if (ctx->device_draw) DEF_HIP(def_launch_ctl_set(ctx->ctl, DEF_CTL_T, t, 0, -1, ctx->stream));
    ctx->t = t;
    return DEF_OK;
}

int def_get_step(const def_ctx *ctx, uint64_t *t)
{
    if (!ctx || !t) return DEF_EINVAL;
    *t = ctx->t;
    return DEF_OK;
}

int def_force_next_start(def_ctx *ctx, int64_t s)
{
    if (!ctx) return DEF_EINVAL;
    if (s >= 0 && (uint64_t)s >= ctx->d) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    if (ctx->device_draw)
        DEF_HIP(def_launch_ctl_set(ctx->ctl, DEF_CTL_FORCED, 0, 0, s < 0 ? -1 : s, ctx->stream));
    ctx->forced = s < 0 ? -1 : s;
    return DEF_OK;
}

int def_last_block(const def_ctx *ctx, uint64_t *start, uint64_t *len)
{
    if (!ctx || !ctx->has_last) return DEF_EINVAL;
    if (start) *start = ctx->last_start;
    if (len) *len = ctx->B;
    return DEF_OK;
}

int def_block_length(const def_ctx *ctx, uint64_t *len)
{
    if (!ctx || !len) return DEF_EINVAL;
    *len = ctx->B;
    return DEF_OK;
}

int def_state_ptrs(def_ctx *ctx, float **e, float **m, float **avg_block, uint64_t *ld_state)
{
    if (!ctx) return DEF_EINVAL;
    if (e) *e = ctx->e;
    if (m) *m = ctx->m;
    if (avg_block) *avg_block = ctx->avg;
    if (ld_state) *ld_state = ctx->ld;
    return DEF_OK;
}

int def_last_path(const def_ctx *ctx, int *flat)
{
    if (!ctx || !flat || !ctx->has_last) return DEF_EINVAL;
    *flat = ctx->last_flat;
    return DEF_OK;
}

const char *def_last_kernel(const def_ctx *ctx)
{
    return ctx && ctx->has_last ? ctx->kernel_name : nullptr;
}

int def_profile_begin(def_ctx *ctx, uint32_t max_steps)
{
    if (!ctx || max_steps == 0 || max_steps > (1u << 20)) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    for (hipEvent_t ev : ctx->ev) (void)hipEventDestroy(ev);
    ctx->ev.clear();
    ctx->prof_cap = ctx->prof_n = 0;
    try {
        ctx->ev.reserve(2 * (size_t)max_steps);
    } catch (const std::bad_alloc &) {
        return DEF_ENOMEM;
    }
    for (uint32_t q = 0; q < 2 * max_steps; ++q) {
        hipEvent_t ev;
        DEF_HIP(hipEventCreate(&ev));
        ctx->ev.push_back(ev);
    }
    ctx->prof_cap = max_steps;
    return DEF_OK;
}

int def_profile_end(def_ctx *ctx, float *ms, uint32_t cap, uint32_t *n)
{
    if (!ctx || !n || (cap && !ms)) return DEF_EINVAL;
    DEF_ON_DEVICE(ctx);
    const uint32_t recorded = ctx->prof_n;
    int rc = DEF_OK;
    if (recorded) {
        hipError_t err = hipEventSynchronize(ctx->ev[2 * recorded - 1]);
        for (uint32_t q = 0; err == hipSuccess && q < recorded && q < cap; ++q)
            err = hipEventElapsedTime(&ms[q], ctx->ev[2 * q], ctx->ev[2 * q + 1]);
        if (err != hipSuccess) rc = hip_fail(err);
    }
    for (hipEvent_t ev : ctx->ev) (void)hipEventDestroy(ev);
    ctx->ev.clear();
    ctx->prof_cap = ctx->prof_n = 0;
    *n = recorded;
    return rc;
}

const char *def_strerror(int status)
{
    switch (status) {
    case DEF_OK: return "ok";
    case DEF_EINVAL: return "invalid argument";
    case DEF_ENOMEM: return "out of memory";
    case DEF_EHIP: return "HIP runtime error (see def_last_hip_error)";
    case DEF_ELIMIT: return "problem larger than the fixed limit of this entry point";
    default: return "unknown status";
    }
}

int def_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
