// C ABI of libkvsched: argument checks, context and scratch management, kernel sequencing.
// All arithmetic of the method runs in the kernels of simulate.hip and sortedf.hip.
#include "kvsched_internal.h"

#include <mutex>
#include <new>

// Working memory of kvsched_best_neighbor_static: a fixed array in the library's device image, so
// that the call needs no allocation.  Every GPU the library is used on holds its own copy at its
// own address; host code never uses the array's name as an address but asks the runtime for it,
// once per device (static_scratch_of_current_device), and passes that pointer on.
constexpr size_t KVS_STATIC_SCRATCH_BYTES = (size_t)KVSCHED_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[KVS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_scratch[kMaxDevices];  // device address of `scratch` on each GPU, once resolved

// Address of this library's `scratch` array on the device that is current (call after hipSetDevice).
int static_scratch_of_current_device(int device, void **out)
{
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return KVSCHED_ERANGE;
    std::lock_guard<std::mutex> guard(g_static_mu);
    if (!g_static_scratch[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KVSCHED_EHIP;
        g_static_scratch[device] = p;
    }
    *out = g_static_scratch[device];
    return KVSCHED_OK;
}

constexpr int64_t kMaxM = (int64_t)1 << 30;
constexpr int32_t WAVE_POSITIONS = 64;  // positions of an order a wavefront fetches at a time
constexpr size_t kMaxExactTableBytes = (size_t)16 << 30;  // tables + records of the exact DP

int ensure_scratch(kvsched_ctx *ctx, size_t bytes)
{
    ctx->resume_rows = 0;  // whoever asks for scratch overwrites the last resume plan
    ctx->rejoin_offset = 0;
    ctx->neighbor_stop_offset = 0;
    if (bytes <= ctx->scratch_bytes) return KVSCHED_OK;
    if (ctx->d_scratch) {
        // kernels of earlier calls may still be reading the old buffer
        if (hipDeviceSynchronize() != hipSuccess) return KVSCHED_EHIP;
        (void)hipFree(ctx->d_scratch);
        ctx->d_scratch = nullptr;
        ctx->scratch_bytes = 0;
    }
    size_t cap = (bytes + ((size_t)1 << 20)) & ~(((size_t)1 << 20) - 1);
    if (hipMalloc(&ctx->d_scratch, cap) != hipSuccess) return KVSCHED_ENOMEM;
    ctx->scratch_bytes = cap;
    return KVSCHED_OK;
}

int ensure_tables(kvsched_ctx *ctx, size_t bytes)
{
    if (bytes <= ctx->tables_bytes) return KVSCHED_OK;
    if (ctx->d_tables) {
        if (hipDeviceSynchronize() != hipSuccess) return KVSCHED_EHIP;
        (void)hipFree(ctx->d_tables);
        ctx->d_tables = nullptr;
        ctx->tables_bytes = 0;
    }
    size_t cap = (bytes + ((size_t)1 << 20)) & ~(((size_t)1 << 20) - 1);
    if (hipMalloc(&ctx->d_tables, cap) != hipSuccess) return KVSCHED_ENOMEM;
    ctx->tables_bytes = cap;
    return KVSCHED_OK;
}

// Read the context's device words back (one stream synchronisation).
int read_words(kvsched_ctx *ctx, hipStream_t st)
{
    if (hipMemcpyAsync(ctx->h_words, ctx->d_words, sizeof(int32_t) * KVS_W_COUNT, hipMemcpyDeviceToHost, st) !=
        hipSuccess)
        return KVSCHED_EHIP;
    return hipStreamSynchronize(st) == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

// The timeline kernel, bracketed by the context's events when timing is on.
int run_timelines(kvsched_ctx *ctx, const SimParams &p, int32_t H, hipStream_t st)
{
    if (ctx->timing && hipEventRecord(ctx->ev0, st) != hipSuccess) return KVSCHED_EHIP;
    // profile in registers when the longest decode fits there, else the LDS ring
    int rc = p.o_bound <= KVS_REG_MAX_O ? kvs_launch_simulate_reg(p, st) : kvs_launch_simulate(p, H, st);
    if (rc != KVSCHED_OK) return rc;
    if (ctx->timing) {
        if (hipEventRecord(ctx->ev1, st) != hipSuccess) return KVSCHED_EHIP;
        ctx->timed = 1;
    }
    return KVSCHED_OK;
}

int32_t ring_slots_for(int32_t o_max)
{
    int32_t h = 64;
    while (h < o_max) h <<= 1;
    return h;
}

// Enqueue the length scan; unless the caller supplied a bound, wait for the largest decode
// length.  *o_bound_out is what the timeline kernels size their ring from.
int scan_and_bound(kvsched_ctx *ctx, const int32_t *s, const int32_t *o, int32_t n, int64_t M, hipStream_t st,
                   int32_t *o_bound_out, const int32_t *moves = nullptr, int32_t K = 0,
                   int32_t *min_position_out = nullptr, int32_t *max_position_out = nullptr)
{
    if (max_position_out) *max_position_out = n - 1;
    int rc = kvs_launch_scan_lengths(s, o, n, (int32_t)M, ctx->o_max_bound, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    if (min_position_out) *min_position_out = 0;
    if (ctx->o_max_bound > 0) {
        *o_bound_out = ctx->o_max_bound;
        return KVSCHED_OK;
    }
    if (moves && min_position_out) {  // rides on the same read-back: first position any move touches
        rc = kvs_launch_moves_min_position(moves, K, n, ctx->d_words, st);
        if (rc != KVSCHED_OK) return rc;
    }
    if (hipMemcpyAsync(ctx->h_words, ctx->d_words, sizeof(int32_t) * KVS_W_COUNT, hipMemcpyDeviceToHost, st) !=
        hipSuccess)
        return KVSCHED_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return KVSCHED_EHIP;
    int32_t omax = ctx->h_words[KVS_W_OMAX];
    if (omax > KVSCHED_MAX_O) return KVSCHED_ERANGE;
    *o_bound_out = omax < 1 ? 1 : omax;
    if (moves && min_position_out) {
        const int32_t mp = ctx->h_words[KVS_W_MINPOS];
        *min_position_out = (mp < 0 || mp > n) ? 0 : mp;  // INT_MAX: no move changes the order
        if (mp == INT32_MAX) *min_position_out = n;
        if (max_position_out) {
            const int32_t top = ctx->h_words[KVS_W_MAXPOS];
            *max_position_out = (top < 0 || top >= n) ? n - 1 : top;
        }
    }
    return KVSCHED_OK;
}

constexpr int32_t kMinSharedPrefix = 64;  // shorter shared prefixes are not worth a launch
// Resuming rows from snapshots of row 0 costs the plan (which rows share what with row 0, sorted:
// some 60 us for 16384 rows) and the wait for row 0's wave; it pays when there is enough work to
// skip.  Measured on random one-swap neighbours of a base order, whole call, no resume / resumed in
// one launch: n = 2000: 4096 rows 1.02 / 0.96 ms, 8192 rows 1.63 / 1.33, 16384 rows 2.96 / 2.25;
// n = 500: 8192 rows 0.42 / 0.41, 16384 rows 0.74 / 0.69; n = 200: never (0.33 / 0.40 at 16384 rows).
// Hence, unless the caller sets a row threshold of his own: at least 4096 rows, 6 blocks of 64
// positions and 8 million positions in all.  In two launches (the quarter of the rows that shares least,
// at most half a chip's worth, from the start next to row 0, then the others) the first launch lasts
// a whole timeline whatever it holds: that pays from 16384 rows on (n = 2000: 2.96 / 2.53 ms).
constexpr int32_t kResumeAutoMinRows = 4096;
constexpr int32_t kResumeAutoMinRowsTwoLaunches = 16384;
constexpr int32_t kResumeAutoMinBlocks = 6;
constexpr int64_t kResumeAutoMinPositions = 8000000;
constexpr int32_t kResumeFirstLaunchMax = 4096;
constexpr int32_t kResumeWaitPollsDefault = 4096;  // about 14 ms
// Streams of kvsched_online run one per wavefront, at most some 1500 to 3000 at once on 256 compute
// units (LDS-limited): below that every stream starts at once and their order is of no consequence.
constexpr int32_t kOnlineOrderMinStreams = 1024;

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }
size_t neighbor_scratch_bytes(int32_t K, int32_t n, int32_t o_bound);

// Are C timelines of n positions to be resumed from the states of the first of them?
static bool resume_pays(const kvsched_ctx *ctx, int32_t C, int32_t n, int32_t o_bound)
{
    if (n <= 2 * WAVE_POSITIONS || o_bound > KVS_REG_MAX_O) return false;
    if (ctx->resume_min_rows != KVSCHED_RESUME_AUTO) return ctx->resume_min_rows > 0 && C >= ctx->resume_min_rows;
    return (n - 1) / WAVE_POSITIONS >= kResumeAutoMinBlocks && (int64_t)C * (int64_t)n >= kResumeAutoMinPositions &&
           C >= (ctx->resume_wait_polls > 0 ? kResumeAutoMinRows : kResumeAutoMinRowsTwoLaunches);
}

__global__ void kvs_copy_i32(int32_t *dst, const int32_t *src, int32_t n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void kvs_fill_zero_i32(int32_t *dst, int32_t n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0;
}
size_t state_bytes() { return align256(sizeof(int32_t) * KVS_STATE_MAX_WORDS); }

// The horizon step's own buffer (kept between steps): state | order copy | s copy | o copy | completion by position | flag.
struct HorizonBuffers {
    int32_t *state, *order, *s, *o, *comp_pos, *ok;
};

size_t horizon_row_bytes(int32_t n) { return align256(sizeof(int32_t) * (size_t)n); }

HorizonBuffers horizon_buffers(kvsched_ctx *ctx, int32_t n)
{
    char *b = (char *)ctx->d_horizon;
    const size_t row = horizon_row_bytes(n);
    HorizonBuffers h;
    h.state = (int32_t *)b;
    h.order = (int32_t *)(b + state_bytes());
    h.s = (int32_t *)(b + state_bytes() + row);
    h.o = (int32_t *)(b + state_bytes() + 2 * row);
    h.comp_pos = (int32_t *)(b + state_bytes() + 3 * row);
    h.ok = (int32_t *)(b + state_bytes() + 4 * row);
    return h;
}

// (growing it forgets what was kept)
int ensure_horizon(kvsched_ctx *ctx, int32_t n)
{
    const size_t bytes = state_bytes() + 4 * horizon_row_bytes(n) + 256;
    if (bytes <= ctx->horizon_bytes) return KVSCHED_OK;
    ctx->hz_len = 0;
    if (ctx->d_horizon) {
        if (hipDeviceSynchronize() != hipSuccess) return KVSCHED_EHIP;
        (void)hipFree(ctx->d_horizon);
        ctx->d_horizon = nullptr;
        ctx->horizon_bytes = 0;
    }
    if (hipMalloc(&ctx->d_horizon, bytes) != hipSuccess) return KVSCHED_ENOMEM;
    ctx->horizon_bytes = bytes;
    return KVSCHED_OK;
}


// Run positions [0, cp) of `row0` once and leave the timeline state in `state`;
// completion rounds of those positions (position order) go to prefix_completion if not NULL.
// prefix_completion: completion rounds of the prefix, by position (by_id = 0: an array of cp entries) or by
// request id (by_id = 1: a row of n entries of which the prefix's requests are written), or null.
// from_len > 0: state holds the timeline after the first from_len positions; they are skipped if *resume_ok != 0.
int run_shared_prefix(const int32_t *row0, int32_t cp, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                      int32_t o_bound, int32_t *d_words, int32_t *state, int32_t *prefix_completion, hipStream_t st,
                      int by_id = 0, int32_t from_len = 0, const int32_t *resume_ok = nullptr)
{
    SimParams q;
    q.src.orders = row0;
    q.src.base = nullptr;
    q.src.moves = nullptr;
    q.C = 1;
    q.n = n;
    q.s = s;
    q.o = o;
    q.M = (int32_t)M;
    q.tel_out = nullptr;
    q.completion_out = prefix_completion;
    q.completion_by_position = by_id ? 0 : 1;
    q.d_words = d_words;
    q.o_bound = o_bound;
    q.k_begin = 0;
    q.k_end = cp;
    q.state_out = state;
    if (from_len > 0 && resume_ok) {
        q.k_begin = from_len;
        q.state_in = state;
        q.resume_ok = resume_ok;
    }
    return kvs_launch_simulate_reg(q, st);
}

int check_common(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M)
{
    if (!ctx || !s || !o || n < 1 || M < 1) return KVSCHED_EINVAL;
    if (M >= kMaxM) return KVSCHED_ERANGE;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    return KVSCHED_OK;
}

}  // namespace

extern "C" {

int kvsched_create(kvsched_ctx **out, int device_id)
{
    if (!out) return KVSCHED_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess) return KVSCHED_EHIP;
    if (device_id < 0 || device_id >= count) return KVSCHED_EINVAL;
    if (hipSetDevice(device_id) != hipSuccess) return KVSCHED_EHIP;
    kvsched_ctx *ctx = new (std::nothrow) kvsched_ctx();
    if (!ctx) return KVSCHED_ENOMEM;
    ctx->device = device_id;
    ctx->o_max_bound = 0;
    ctx->d_words = nullptr;
    ctx->h_words = nullptr;
    ctx->d_scratch = nullptr;
    ctx->scratch_bytes = 0;
    ctx->static_scratch = nullptr;
    ctx->d_tables = nullptr;
    ctx->tables_bytes = 0;
    ctx->d_horizon = nullptr;
    ctx->horizon_bytes = 0;
    ctx->hz_n = ctx->hz_len = ctx->hz_o_bound = 0;
    ctx->hz_M = 0;
    ctx->timing = 0;
    ctx->timed = 0;
    ctx->resume_rows = 0;
    ctx->rejoin_offset = 0;
    ctx->neighbor_stop_offset = 0;
    ctx->neighbor_moves = 0;
    ctx->resume_first = 0;
    ctx->resume_min_rows = KVSCHED_RESUME_AUTO;
    ctx->resume_wait_polls = kResumeWaitPollsDefault;
    ctx->ev0 = nullptr;
    ctx->ev1 = nullptr;
    if (hipMalloc((void **)&ctx->d_words, sizeof(int32_t) * KVS_W_COUNT) != hipSuccess ||
        hipHostMalloc((void **)&ctx->h_words, sizeof(int32_t) * KVS_W_COUNT, hipHostMallocDefault) != hipSuccess ||
        hipMemset(ctx->d_words, 0, sizeof(int32_t) * KVS_W_COUNT) != hipSuccess) {
        kvsched_destroy(ctx);
        return KVSCHED_ENOMEM;
    }
    // devices beyond the table simply cannot use kvsched_best_neighbor_static
    if (device_id < kMaxDevices) {
        const int rc = static_scratch_of_current_device(device_id, &ctx->static_scratch);
        if (rc != KVSCHED_OK) {
            kvsched_destroy(ctx);
            return rc;
        }
    }
    *out = ctx;
    return KVSCHED_OK;
}

void kvsched_destroy(kvsched_ctx *ctx)
{
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    if (ctx->d_words) (void)hipFree(ctx->d_words);
    if (ctx->h_words) (void)hipHostFree(ctx->h_words);
    if (ctx->d_scratch) (void)hipFree(ctx->d_scratch);
    if (ctx->d_tables) (void)hipFree(ctx->d_tables);
    if (ctx->d_horizon) (void)hipFree(ctx->d_horizon);
    if (ctx->ev0) (void)hipEventDestroy(ctx->ev0);
    if (ctx->ev1) (void)hipEventDestroy(ctx->ev1);
    delete ctx;
}

const char *kvsched_strerror(int status)
{
    switch (status) {
        case KVSCHED_OK: return "ok";
        case KVSCHED_EINVAL: return "invalid argument (null pointer, non-positive size or bad enum)";
        case KVSCHED_ERANGE: return "size outside the supported range";
        case KVSCHED_EHIP: return "HIP runtime call failed";
        case KVSCHED_ENOMEM: return "out of device or host memory";
        default: return "unknown status";
    }
}

int kvsched_reserve(kvsched_ctx *ctx, int32_t rows, int32_t n, int32_t moves)
{
    if (!ctx || rows < 0 || n < 1 || moves < 0) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    // the largest of what the calls named in the header ask of the scratch buffer at these sizes
    const size_t nblk = (size_t)((n - 1) / WAVE_POSITIONS);
    const size_t row_bytes = align256(sizeof(int32_t) * (size_t)n);
    size_t need = kvs_sortedF_scratch_bytes(n);
    const size_t swap = kvs_local_swap_scratch_bytes(n);
    if (swap > need) need = swap;
    if (rows > 0) {
        const size_t sim = 6 * align256(sizeof(int32_t) * (size_t)rows) +
                           align256(sizeof(int32_t) * nblk * KVS_STATE_MAX_WORDS) +
                           align256(sizeof(int32_t) * KVS_PROGRESS_WORDS) + 2 * row_bytes;
        const size_t pre = state_bytes() + row_bytes;  // a declared common prefix
        if (sim > need) need = sim;
        if (pre > need) need = pre;
    }
    if (moves > 0) {
        const size_t hor = neighbor_scratch_bytes(moves, n, ctx->o_max_bound) + 2 * row_bytes + 256;
        if (hor > need) need = hor;
    }
    const int32_t keep = ctx->resume_rows;  // reserving is no call: the last resume plan stays readable unless the buffer moves
    const size_t keep_rejoin = ctx->rejoin_offset;
    const bool grows = need > ctx->scratch_bytes;
    const int rc = ensure_scratch(ctx, need);
    if (!grows) ctx->resume_rows = keep, ctx->rejoin_offset = keep_rejoin;
    return rc;
}

int kvsched_set_o_max(kvsched_ctx *ctx, int32_t o_max_bound)
{
    if (!ctx || o_max_bound < 0) return KVSCHED_EINVAL;
    if (o_max_bound > KVSCHED_MAX_O) return KVSCHED_ERANGE;
    ctx->o_max_bound = o_max_bound;
    return KVSCHED_OK;
}

int kvsched_set_resume_one_launch(kvsched_ctx *ctx, int32_t wait_polls)
{
    if (!ctx || wait_polls < 0) return KVSCHED_EINVAL;
    ctx->resume_wait_polls = wait_polls;
    return KVSCHED_OK;
}

int kvsched_set_resume_min_rows(kvsched_ctx *ctx, int32_t rows)
{
    if (!ctx || (rows < 0 && rows != KVSCHED_RESUME_AUTO)) return KVSCHED_EINVAL;
    ctx->resume_min_rows = rows;
    return KVSCHED_OK;
}

int kvsched_enable_timing(kvsched_ctx *ctx, int on)
{
    if (!ctx) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    if (on && !ctx->ev0) {
        if (hipEventCreate(&ctx->ev0) != hipSuccess || hipEventCreate(&ctx->ev1) != hipSuccess) return KVSCHED_EHIP;
    }
    ctx->timing = on ? 1 : 0;
    ctx->timed = 0;
    return KVSCHED_OK;
}

int kvsched_last_timeline_ms(kvsched_ctx *ctx, float *ms_out)
{
    if (!ctx || !ms_out || !ctx->timing || !ctx->timed) return KVSCHED_EINVAL;
    if (hipEventSynchronize(ctx->ev1) != hipSuccess) return KVSCHED_EHIP;
    if (hipEventElapsedTime(ms_out, ctx->ev0, ctx->ev1) != hipSuccess) return KVSCHED_EHIP;
    return KVSCHED_OK;
}

int kvsched_device_status(kvsched_ctx *ctx, void *stream, int32_t *status_out)
{
    if (!ctx || !status_out) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(ctx->h_words, ctx->d_words, sizeof(int32_t) * KVS_W_COUNT, hipMemcpyDeviceToHost, st) !=
        hipSuccess)
        return KVSCHED_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return KVSCHED_EHIP;
    *status_out = ctx->h_words[KVS_W_STATUS];
    return KVSCHED_OK;
}

int kvsched_simulate(kvsched_ctx *ctx, const int32_t *orders, int32_t C, int32_t n, const int32_t *s,
                     const int32_t *o, int64_t M, int64_t *tel_out, int32_t *completion_out, int32_t common_prefix,
                     void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!orders || !tel_out || C < 1 || common_prefix < 0 || common_prefix > n) return KVSCHED_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    int32_t o_bound = 0;
    rc = scan_and_bound(ctx, s, o, n, M, st, &o_bound);
    if (rc != KVSCHED_OK) return rc;
    const int32_t H = ring_slots_for(o_bound);
    if ((int64_t)n * (int64_t)H >= kMaxM) return KVSCHED_ERANGE;  // rounds are int32
    SimParams p;
    p.src.orders = orders;
    p.src.base = nullptr;
    p.src.moves = nullptr;
    p.C = C;
    p.n = n;
    p.s = s;
    p.o = o;
    p.M = (int32_t)M;
    p.tel_out = tel_out;
    p.completion_out = completion_out;
    // Completion rounds leave the timeline kernel in position order (coalesced stores); a second
    // kernel permutes each row to request-id order through LDS.  Rows too long for LDS are
    // scattered by the timeline kernel itself.
    p.completion_by_position = (completion_out && n <= KVS_PERMUTE_MAX_N) ? 1 : 0;
    p.d_words = ctx->d_words;
    p.o_bound = o_bound;
    // Declared common prefix: run it once (row 0), resume every row from its state.
    int32_t cp = 0;
    int32_t *prefix_comp = nullptr;
    if (common_prefix >= kMinSharedPrefix && C > 1 && o_bound <= KVS_REG_MAX_O &&
        (!completion_out || p.completion_by_position)) {
        cp = common_prefix;
        rc = ensure_scratch(ctx, state_bytes() + align256(sizeof(int32_t) * (size_t)cp));
        if (rc != KVSCHED_OK) return rc;
        int32_t *state = (int32_t *)ctx->d_scratch;
        if (completion_out) prefix_comp = (int32_t *)((char *)ctx->d_scratch + state_bytes());
        rc = run_shared_prefix(orders, cp, n, s, o, M, o_bound, ctx->d_words, state, prefix_comp, st);
        if (rc != KVSCHED_OK) return rc;
        p.k_begin = cp;
        p.state_in = state;
    }
    // No declared prefix: rows that agree with row 0 on their leading 64-position blocks resume
    // from snapshots of row 0's timeline, taken by row 0's own wave.
    ctx->resume_rows = 0;
    ctx->rejoin_offset = 0;
    const int32_t *resumed_blocks = nullptr, *resumed_row0 = nullptr, *rejoined = nullptr;
    if (cp == 0 && resume_pays(ctx, C, n, o_bound)) {
        const int32_t nblk = (n - 1) / WAVE_POSITIONS;
        const int32_t stride = kvs_reg_state_words(o_bound);
        const size_t list_bytes = align256(sizeof(int32_t) * (size_t)C);
        const size_t snap_bytes = align256(sizeof(int32_t) * (size_t)nblk * (size_t)stride);
        const size_t flag_bytes = align256(sizeof(int32_t) * KVS_PROGRESS_WORDS);  // the progress word of row 0's wave
        const size_t row_bytes = align256(sizeof(int32_t) * (size_t)n);
        rc = ensure_scratch(ctx, 6 * list_bytes + snap_bytes + flag_bytes + 2 * row_bytes);
        if (rc != KVSCHED_OK) return rc;
        int32_t *blocks = (int32_t *)ctx->d_scratch;
        int32_t *sorted = (int32_t *)((char *)ctx->d_scratch + list_bytes);
        int32_t *tmp = (int32_t *)((char *)ctx->d_scratch + 2 * list_bytes);
        int32_t *snaps = (int32_t *)((char *)ctx->d_scratch + 3 * list_bytes);
        int32_t *flags = (int32_t *)((char *)ctx->d_scratch + 3 * list_bytes + snap_bytes);
        int32_t *row0 = (int32_t *)((char *)ctx->d_scratch + 3 * list_bytes + snap_bytes + flag_bytes);
        // A row may also stop before its end, where its timeline has become row 0's again (see SimParams);
        // not when the timeline kernel itself scatters the completion rounds by request id.
        const bool rejoin = !completion_out || p.completion_by_position;
        char *more = (char *)ctx->d_scratch + 3 * list_bytes + snap_bytes + flag_bytes + row_bytes;
        int32_t *diff_first = (int32_t *)more, *diff_last = (int32_t *)(more + list_bytes);
        int32_t *rejoin_block = (int32_t *)(more + 2 * list_bytes);
        int32_t *start0 = (int32_t *)(more + 3 * list_bytes);
        rc = kvs_launch_shared_blocks(orders, C, n, blocks, rejoin ? diff_first : nullptr, diff_last, st);
        if (rc != KVSCHED_OK) return rc;
        if (rejoin) {
            p.diff_first = diff_first;
            p.diff_last = diff_last;
            p.rejoin_block = rejoin_block;
            p.start0 = start0;
        }
        rc = kvs_launch_sort_by_blocks(blocks, C, 0, tmp, sorted, flags, KVS_PROGRESS_WORDS, st);  // (clears the progress word too)
        if (rc != KVSCHED_OK) return rc;
        int32_t first = 0;
        if (ctx->resume_wait_polls > 0) {
            // All rows in one launch, those that share least with row 0 first: row 0's wave reports each
            // snapshot as it is written, the others wait for theirs (most find it there already).
            if (ctx->timing && hipEventRecord(ctx->ev0, st) != hipSuccess) return KVSCHED_EHIP;
            SimParams a = p;
            a.cand_list = sorted;
            a.resume_block = blocks;
            a.snapshots = snaps;
            a.snap_stride = stride;
            a.snap_blocks = nblk;
            a.snap_flags = flags;
            a.snap_wait_polls = ctx->resume_wait_polls;
            a.rejoin_blocks = rejoin ? nblk : 0;
            rc = kvs_launch_simulate_reg(a, st);
            if (rc != KVSCHED_OK) return rc;
        } else {
            rc = kvs_launch_mark_snapshots_unusable(snaps, nblk, stride, st);
            if (rc != KVSCHED_OK) return rc;
            first = (C + 3) / 4 < kResumeFirstLaunchMax ? (C + 3) / 4 : kResumeFirstLaunchMax;
            if (ctx->timing && hipEventRecord(ctx->ev0, st) != hipSuccess) return KVSCHED_EHIP;
            SimParams a = p;  // rows sorted[0 .. first): from the start; row 0 (sorted[0]) takes the snapshots
            a.C = first;
            a.cand_list = sorted;
            a.snapshots = snaps;
            a.snap_stride = stride;
            a.snap_blocks = nblk;
            rc = kvs_launch_simulate_reg(a, st);
            if (rc != KVSCHED_OK) return rc;
            SimParams b = p;  // rows sorted[first .. C): from their snapshot
            b.C = C - first;
            b.cand_list = sorted + first;
            b.resume_block = blocks;
            b.snapshots = snaps;
            b.snap_stride = stride;
            b.snap_blocks = 0;
            b.rejoin_blocks = rejoin ? nblk : 0;  // (the first launch has left every state and start round of row 0)
            rc = kvs_launch_simulate_reg(b, st);
            if (rc != KVSCHED_OK) return rc;
        }
        if (rejoin) {
            rc = kvs_launch_rejoin_finish(rejoin_block, C, 0, tel_out, st);
            if (rc != KVSCHED_OK) return rc;
            rejoined = rejoin_block;
            ctx->rejoin_offset = (size_t)((char *)rejoin_block - (char *)ctx->d_scratch);
        }
        if (ctx->timing) {
            if (hipEventRecord(ctx->ev1, st) != hipSuccess) return KVSCHED_EHIP;
            ctx->timed = 1;
        }
        if (completion_out && p.completion_by_position) {
            // the permute pass takes the positions a row did not place from this copy of row 0's row
            hipLaunchKernelGGL(kvs_copy_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, row0, completion_out, n);
            if (hipGetLastError() != hipSuccess) return KVSCHED_EHIP;
            resumed_blocks = blocks;
            resumed_row0 = row0;
        } else if (completion_out) {
            rc = kvs_launch_copy_row0_prefix(orders, C, n, sorted, first, blocks, p.completion_by_position,
                                             completion_out, st);
            if (rc != KVSCHED_OK) return rc;
        }
        ctx->resume_rows = C;
        ctx->resume_first = first;
    } else {
        rc = run_timelines(ctx, p, H, st);
        if (rc != KVSCHED_OK) return rc;
    }
    if (prefix_comp) {
        rc = kvs_launch_broadcast_prefix(prefix_comp, cp, C, n, completion_out, st);
        if (rc != KVSCHED_OK) return rc;
    }
    if (p.completion_by_position) {  // this pass over the rows checks them as well
        rc = kvs_launch_permute_rows(orders, C, n, completion_out, tel_out, ctx->d_words, resumed_blocks, resumed_row0,
                                     resumed_row0 ? rejoined : nullptr, st);
    } else {
        rc = kvs_launch_check_orders(orders, C, n, tel_out, ctx->d_words, st);
    }
    if (rc != KVSCHED_OK || cp == 0) return rc;
    return kvs_launch_check_prefix(orders, C, n, cp, tel_out, ctx->d_words, st);
}

// The three Phase-1 solvers; (ga, gb) = (0, 1) is the F-metric.
static int run_sortedF(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t ga,
                       int32_t gb, int32_t tie_rule, int32_t feas_mode, int32_t *order_out, int32_t *batch_end_out,
                       double *F_out, int32_t *num_batches_out, void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!order_out || !batch_end_out || !F_out || !num_batches_out) return KVSCHED_EINVAL;
    if (tie_rule != KVSCHED_TIE_LARGER && tie_rule != KVSCHED_TIE_SMALLER) return KVSCHED_EINVAL;
    if (feas_mode != KVSCHED_FEAS_SUM_OF_PEAKS && feas_mode != KVSCHED_FEAS_PROFILE) return KVSCHED_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    rc = ensure_scratch(ctx, kvs_sortedF_scratch_bytes(n));
    if (rc != KVSCHED_OK) return rc;
    rc = kvs_launch_scan_lengths(s, o, n, (int32_t)M, 0, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    return kvs_launch_sortedF(n, s, o, (int32_t)M, ga, gb, tie_rule, feas_mode, order_out, batch_end_out, F_out,
                              num_batches_out, ctx->d_scratch, ctx->d_words, st);
}

int kvsched_sortedF(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t tie_rule,
                    int32_t feas_mode, int32_t *order_out, int32_t *batch_end_out, double *F_out,
                    int32_t *num_batches_out, void *stream)
{
    return run_sortedF(ctx, n, s, o, M, 0, 1, tie_rule, feas_mode, order_out, batch_end_out, F_out, num_batches_out,
                       stream);
}

static int run_local_swap(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t ga,
                          int32_t gb, int32_t *order_out, int32_t *batch_end_out, double *F_out, int32_t *swaps_out,
                          int32_t *num_batches_out, void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!order_out || !batch_end_out || !F_out || !num_batches_out) return KVSCHED_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    rc = ensure_scratch(ctx, kvs_local_swap_scratch_bytes(n));
    if (rc != KVSCHED_OK) return rc;
    rc = kvs_launch_scan_lengths(s, o, n, (int32_t)M, 0, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    return kvs_launch_local_swap(n, s, o, (int32_t)M, ga, gb, order_out, batch_end_out, F_out, swaps_out,
                                 num_batches_out, ctx->d_scratch, ctx->d_words, st);
}

int kvsched_local_swap(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                       int32_t *order_out, int32_t *batch_end_out, double *F_out, int32_t *swaps_out,
                       int32_t *num_batches_out, void *stream)
{
    return run_local_swap(ctx, n, s, o, M, 0, 1, order_out, batch_end_out, F_out, swaps_out, num_batches_out, stream);
}

static int run_exact_dp(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t ga,
                        int32_t gb, int32_t feas_mode, int32_t tie_rule, int32_t *order_out, int32_t *batch_end_out,
                        double *F_out, int32_t *num_batches_out, void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!order_out || !batch_end_out || !F_out || !num_batches_out) return KVSCHED_EINVAL;
    if (tie_rule != KVSCHED_TIE_LARGER && tie_rule != KVSCHED_TIE_SMALLER) return KVSCHED_EINVAL;
    if (feas_mode != KVSCHED_FEAS_SUM_OF_PEAKS && feas_mode != KVSCHED_FEAS_PROFILE) return KVSCHED_EINVAL;
    if (n > KVSCHED_EXACT_MAX_N) return KVSCHED_ERANGE;
    hipStream_t st = (hipStream_t)stream;
    rc = ensure_scratch(ctx, kvs_exact_dp_list_bytes(n));
    if (rc != KVSCHED_OK) return rc;
    rc = kvs_launch_scan_lengths(s, o, n, (int32_t)M, 0, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    // Small problems run in one workgroup with both tables in LDS; a batch holds at most M / 2
    // requests (each costs at least 2 of the budget), which may already show that they fit.
    const int32_t k_host = (int32_t)((M / 2 < n) ? M / 2 : n);
    if (const int lg = kvs_exact_dp_small_lg(n, k_host, (int32_t)M)) {
        rc = ensure_tables(ctx, kvs_exact_dp_small_record_bytes(n, k_host, lg));
        if (rc != KVSCHED_OK) return rc;
        return kvs_launch_exact_dp_small(n, s, o, (int32_t)M, ga, gb, feas_mode, tie_rule, lg, ctx->d_scratch, ctx->d_tables,
                                         order_out, batch_end_out, F_out, num_batches_out, ctx->d_words, st);
    }
    rc = kvs_launch_exact_dp_prepare(n, s, o, (int32_t)M, feas_mode, ctx->d_scratch, ctx->d_words, num_batches_out, st);
    if (rc != KVSCHED_OK) return rc;
    rc = read_words(ctx, st);
    if (rc != KVSCHED_OK) return rc;
    int32_t r = ctx->h_words[KVS_W_REMAIN], kmax = ctx->h_words[KVS_W_KMAX];
    if (r == 0) return KVSCHED_OK;  // malformed lengths: reported in the device status, no batches
    if (r != n || kmax < 1 || kmax > n) return KVSCHED_EHIP;
    if (const int lg = kvs_exact_dp_small_lg(n, kmax, (int32_t)M)) {  // fits after all, with the true bound
        rc = ensure_tables(ctx, kvs_exact_dp_small_record_bytes(n, kmax, lg));
        if (rc != KVSCHED_OK) return rc;
        return kvs_launch_exact_dp_small(n, s, o, (int32_t)M, ga, gb, feas_mode, tie_rule, lg, ctx->d_scratch, ctx->d_tables,
                                         order_out, batch_end_out, F_out, num_batches_out, ctx->d_words, st);
    }
    const size_t bytes = kvs_exact_dp_table_bytes(r, kmax, (int32_t)M);
    if (bytes > kMaxExactTableBytes) return KVSCHED_ERANGE;
    rc = ensure_tables(ctx, bytes);
    if (rc != KVSCHED_OK) return rc;
    int32_t nb = 0;
    while (r > 0) {  // r falls by at least one per batch
        rc = kvs_launch_exact_dp_batch(n, r, kmax, s, o, (int32_t)M, ga, gb, feas_mode, tie_rule, nb, ctx->d_scratch,
                                       ctx->d_tables, batch_end_out, F_out, ctx->d_words, st);
        if (rc != KVSCHED_OK) return rc;
        rc = read_words(ctx, st);
        if (rc != KVSCHED_OK) return rc;
        const int32_t r_next = ctx->h_words[KVS_W_REMAIN], k_next = ctx->h_words[KVS_W_KMAX];
        ++nb;
        if (r_next < 0 || r_next >= r || k_next > kmax || (r_next > 0 && k_next < 1)) return KVSCHED_EHIP;
        r = r_next;
        kmax = k_next;
    }
    return kvs_launch_exact_dp_emit(n, nb, ctx->d_scratch, order_out, num_batches_out, st);
}

int kvsched_exact_dp(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t feas_mode,
                     int32_t tie_rule, int32_t *order_out, int32_t *batch_end_out, double *F_out,
                     int32_t *num_batches_out, void *stream)
{
    return run_exact_dp(ctx, n, s, o, M, 0, 1, feas_mode, tie_rule, order_out, batch_end_out, F_out, num_batches_out,
                        stream);
}

int kvsched_phase1_G(kvsched_ctx *ctx, int32_t solver, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                     int32_t alpha_num, int32_t alpha_den, int32_t tie_rule, int32_t feas_mode, int32_t *order_out,
                     int32_t *batch_end_out, double *G_out, int32_t *swaps_out, int32_t *num_batches_out, void *stream)
{
    if (alpha_num < 0 || alpha_den < 1 || M < 1) return KVSCHED_EINVAL;
    // Effective lengths alpha_num s_i + alpha_den o_i <= big (s_i + o_i) <= big M.  The sorted-prefix
    // kernel sums them in int64 (and needs alpha_den k^2 exact in a double); Local Swap Search keeps one
    // per request in an int32; the exact DP keeps sums over a batch in int32 (at most M under the sum of
    // peaks, 2 M under the profile constraint).
    const int64_t big = alpha_num > alpha_den ? alpha_num : alpha_den;
    const int64_t lim = (int64_t)1 << 31;
    if (big > 65535) return KVSCHED_ERANGE;
    if (solver == KVSCHED_SOLVER_LOCAL_SWAP && big * M >= lim) return KVSCHED_ERANGE;
    if (solver == KVSCHED_SOLVER_EXACT_DP && big * 2 * M >= lim) return KVSCHED_ERANGE;
    switch (solver) {
        case KVSCHED_SOLVER_SORTED_PREFIX:
            return run_sortedF(ctx, n, s, o, M, alpha_num, alpha_den, tie_rule, feas_mode, order_out, batch_end_out,
                               G_out, num_batches_out, stream);
        case KVSCHED_SOLVER_LOCAL_SWAP:
            if (feas_mode != KVSCHED_FEAS_SUM_OF_PEAKS) return KVSCHED_EINVAL;
            return run_local_swap(ctx, n, s, o, M, alpha_num, alpha_den, order_out, batch_end_out, G_out, swaps_out,
                                  num_batches_out, stream);
        case KVSCHED_SOLVER_EXACT_DP:
            return run_exact_dp(ctx, n, s, o, M, alpha_num, alpha_den, feas_mode, tie_rule, order_out, batch_end_out,
                                G_out, num_batches_out, stream);
        default: return KVSCHED_EINVAL;
    }
}

// Scratch of kvsched_best_neighbor: K + 1 latencies, the state of a shared prefix, where each move's timeline
// stopped because it had become the base order's again (K + 1 entries) with the base order's start rounds (n),
// and the plan for resuming each move's timeline from the base order's (three lists of K + 1 entries, a flag
// and a saved state of the largest kind per 64 positions).
namespace {
// o_bound: the caller's bound on the decode lengths if there is one (it fixes the size of a saved state), else 0.
size_t neighbor_scratch_bytes(int32_t K, int32_t n, int32_t o_bound)
{
    const size_t nblk = (size_t)((n - 1) / WAVE_POSITIONS);
    const size_t words = o_bound > KVS_REG_MAX_O ? 0  // beyond the register kernel nothing is resumed
                         : o_bound > 0           ? (size_t)kvs_reg_state_words(o_bound)
                                                 : KVS_STATE_MAX_WORDS;
    return align256(sizeof(int64_t) * ((size_t)K + 1)) + state_bytes() +
           4 * align256(sizeof(int32_t) * ((size_t)K + 1)) + align256(sizeof(int32_t) * (size_t)n) +
           align256(sizeof(int32_t) * KVS_PROGRESS_WORDS) + align256(sizeof(int32_t) * nblk * words);
}
}  // namespace

// kvsched_best_neighbor on working memory `work` of at least neighbor_scratch_bytes(K, n) bytes.
// o_bound_known > 0: the caller's bound on the decode lengths; nothing is read back from the device
// (so the lowest position the moves touch is not known either and no common prefix is placed ahead:
// moves far into the order start from the base order's saved states instead).
// For kvsched_horizon_step (keep != nullptr, with prefix_completion_by_id and prefix_len_out): when a common
// prefix is placed ahead, its state is left in the horizon buffers, its requests' completion rounds go to
// prefix_completion_by_id and its length is returned.  If the buffers hold the state of a shorter prefix from
// the step before (ctx->hz_len positions, same n, M and decode bound), the prefix run starts there, provided the
// order up to there and the lengths still equal the copies kept with it (compared on the device).
static int best_neighbor_on(kvsched_ctx *ctx, void *work, int32_t o_bound_known, const int32_t *base_order, int32_t n,
                            const int32_t *moves, int32_t K, const int32_t *s, const int32_t *o, int64_t M,
                            int64_t *tel_out, int64_t *result_out, hipStream_t st,
                            const HorizonBuffers *keep = nullptr, int32_t *prefix_completion_by_id = nullptr,
                            int32_t *prefix_len_out = nullptr)
{
    // work: [K+1] latencies (neighbours, then the base order) | state of the shared prefix | resume plan
    const size_t tel_bytes = align256(sizeof(int64_t) * ((size_t)K + 1));
    int64_t *tel = (int64_t *)work;
    int32_t *state = (int32_t *)((char *)work + tel_bytes);
    const size_t list_bytes_all = align256(sizeof(int32_t) * ((size_t)K + 1));
    int32_t *rejoin_block = (int32_t *)((char *)work + tel_bytes + state_bytes());
    int32_t *start0 = (int32_t *)((char *)work + tel_bytes + state_bytes() + list_bytes_all);
    const size_t plan_offset = tel_bytes + state_bytes() + list_bytes_all + align256(sizeof(int32_t) * (size_t)n);
    int32_t o_bound = 0, min_pos = 0, max_pos = n - 1;
    bool stops_early = false;
    ctx->neighbor_stop_offset = 0;
    int rc;
    if (o_bound_known > 0) {
        rc = kvs_launch_scan_lengths(s, o, n, (int32_t)M, o_bound_known, ctx->d_words, st);
        o_bound = o_bound_known;
    } else {
        rc = scan_and_bound(ctx, s, o, n, M, st, &o_bound, moves, K, &min_pos, &max_pos);
    }
    if (rc != KVSCHED_OK) return rc;
    const int32_t H = ring_slots_for(o_bound);
    if ((int64_t)n * (int64_t)H >= kMaxM) return KVSCHED_ERANGE;
    SimParams p;
    p.src.orders = nullptr;
    p.src.base = base_order;
    p.src.moves = moves;
    p.C = K + 1;
    p.n = n;
    p.s = s;
    p.o = o;
    p.M = (int32_t)M;
    p.tel_out = tel;
    p.completion_out = nullptr;
    p.completion_by_position = 0;
    p.d_words = ctx->d_words;
    p.o_bound = o_bound;
    // No move touches a position before min_pos: that prefix of the base order is common to
    // every neighbour, so it is placed once and all timelines resume from its state.
    if (min_pos >= kMinSharedPrefix && o_bound <= KVS_REG_MAX_O) {
        if (keep) {
            int32_t from = 0;
            if (ctx->hz_len >= kMinSharedPrefix && ctx->hz_len <= min_pos && ctx->hz_n == n && ctx->hz_M == M &&
                ctx->hz_o_bound == o_bound)
                from = ctx->hz_len;
            ctx->hz_len = 0;  // (until this step has left its own)
            rc = kvs_launch_horizon_verify(base_order, s, o, n, from, min_pos, keep->order, keep->s, keep->o, keep->ok, st);
            if (rc != KVSCHED_OK) return rc;
            state = keep->state;
            rc = run_shared_prefix(base_order, min_pos, n, s, o, M, o_bound, ctx->d_words, state, keep->comp_pos, st, 0,
                                   from, keep->ok);
            if (rc != KVSCHED_OK) return rc;
            rc = kvs_launch_scatter_prefix(base_order, keep->comp_pos, min_pos, n, prefix_completion_by_id, st);
            if (rc != KVSCHED_OK) return rc;
            ctx->hz_len = min_pos, ctx->hz_n = n, ctx->hz_M = M, ctx->hz_o_bound = o_bound;
        } else {
            rc = run_shared_prefix(base_order, min_pos, n, s, o, M, o_bound, ctx->d_words, state, nullptr, st);
            if (rc != KVSCHED_OK) return rc;
        }
        p.k_begin = min_pos;
        p.state_in = state;
        if (prefix_len_out) *prefix_len_out = min_pos;
        // A move that only reorders requests the base order starts in one and the same round changes no
        // completion round (see the timeline kernel): the base order is placed once more, alone, through the last
        // position any move touches, and the moves found to be of that kind are not run at all.
        if (min_pos < n && max_pos >= min_pos) {
            SimParams q = p;
            q.src.orders = base_order;
            q.src.base = nullptr;
            q.src.moves = nullptr;
            q.C = 1;
            q.tel_out = nullptr;
            q.k_end = max_pos + 1;
            q.start0 = start0;  // (by position)
            rc = kvs_launch_simulate_reg(q, st);
            if (rc != KVSCHED_OK) return rc;
            rc = kvs_launch_mark_noop_moves(moves, K, n, min_pos, max_pos + 1 - min_pos, start0 + min_pos, state,
                                            rejoin_block, st);
            if (rc != KVSCHED_OK) return rc;
            p.skip = rejoin_block;
            stops_early = true;
        }
    } else if (keep) {
        ctx->hz_len = 0;
    }
    if (!p.state_in && ctx->resume_wait_polls > 0 && resume_pays(ctx, K + 1, n, o_bound)) {
        // Moves anywhere in the order (no prefix common to all): a move at positions i, j leaves the
        // positions before min(i, j) as they are, so its timeline starts from the state the base
        // order's timeline (run in the same launch) has saved at the last 64-position boundary before.
        const int32_t C = K + 1;
        const int32_t nblk = (n - 1) / WAVE_POSITIONS;
        const int32_t stride = kvs_reg_state_words(o_bound);
        const size_t list_bytes = align256(sizeof(int32_t) * (size_t)C);
        char *plan = (char *)work + plan_offset;
        int32_t *blocks = (int32_t *)plan;
        int32_t *sorted = (int32_t *)(plan + list_bytes);
        int32_t *tmp = (int32_t *)(plan + 2 * list_bytes);
        int32_t *flags = (int32_t *)(plan + 3 * list_bytes);
        int32_t *snaps = (int32_t *)(plan + 3 * list_bytes + align256(sizeof(int32_t) * KVS_PROGRESS_WORDS));
        rc = kvs_launch_move_blocks(moves, K, n, blocks, st);
        if (rc != KVSCHED_OK) return rc;
        rc = kvs_launch_sort_by_blocks(blocks, C, K, tmp, sorted, flags, KVS_PROGRESS_WORDS, st);  // (clears the progress word too)
        if (rc != KVSCHED_OK) return rc;
        p.cand_list = sorted;
        p.resume_block = blocks;
        p.snapshots = snaps;
        p.snap_stride = stride;
        p.snap_blocks = nblk;
        p.snap_flags = flags;
        p.snap_wait_polls = ctx->resume_wait_polls;
        p.snap_cand = K;
        p.rejoin_block = rejoin_block;  // a move's timeline stops where it has become the base order's again
        p.start0 = start0;
        p.rejoin_blocks = nblk;
        stops_early = true;
        if (ctx->timing && hipEventRecord(ctx->ev0, st) != hipSuccess) return KVSCHED_EHIP;
        rc = kvs_launch_simulate_reg(p, st);
        if (rc == KVSCHED_OK && ctx->timing) {
            if (hipEventRecord(ctx->ev1, st) != hipSuccess) return KVSCHED_EHIP;
            ctx->timed = 1;
        }
    } else {
        rc = run_timelines(ctx, p, H, st);
    }
    if (rc != KVSCHED_OK) return rc;
    if (stops_early) {
        rc = kvs_launch_rejoin_finish(rejoin_block, K + 1, K, tel, st);
        if (rc != KVSCHED_OK) return rc;
        if (work == ctx->d_scratch) {
            ctx->neighbor_stop_offset = (size_t)((char *)rejoin_block - (char *)work);
            ctx->neighbor_moves = K;
        }
    }
    rc = kvs_launch_check_moves(moves, K, n, tel, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    rc = kvs_launch_check_orders(base_order, 1, n, tel + K, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    rc = kvs_launch_argmin(tel, K, result_out, 1, st);
    if (rc != KVSCHED_OK) return rc;
    if (tel_out &&
        hipMemcpyAsync(tel_out, tel, sizeof(int64_t) * (size_t)K, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return KVSCHED_EHIP;
    return KVSCHED_OK;
}

int kvsched_best_neighbor(kvsched_ctx *ctx, const int32_t *base_order, int32_t n, const int32_t *moves, int32_t K,
                          const int32_t *s, const int32_t *o, int64_t M, int64_t *tel_out, int64_t *result_out,
                          void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!base_order || !moves || !result_out || K < 1 || K == INT32_MAX) return KVSCHED_EINVAL;
    rc = ensure_scratch(ctx, neighbor_scratch_bytes(K, n, ctx->o_max_bound));
    if (rc != KVSCHED_OK) return rc;
    return best_neighbor_on(ctx, ctx->d_scratch, ctx->o_max_bound, base_order, n, moves, K, s, o, M, tel_out,
                            result_out, (hipStream_t)stream);
}

int kvsched_best_neighbor_static(kvsched_ctx *ctx, const int32_t *base_order, int32_t n, const int32_t *moves,
                                 int32_t K, const int32_t *s, const int32_t *o, int64_t M, int32_t o_max_bound,
                                 int64_t *tel_out, int64_t *result_out, void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!base_order || !moves || !result_out || K < 1 || K == INT32_MAX || o_max_bound < 1) return KVSCHED_EINVAL;
    if (o_max_bound > KVSCHED_MAX_O) return KVSCHED_ERANGE;
    if (!ctx->static_scratch) return KVSCHED_ERANGE;  // device number beyond the table of resolved addresses
    if (neighbor_scratch_bytes(K, n, o_max_bound) > KVS_STATIC_SCRATCH_BYTES) return KVSCHED_ERANGE;
    // Nothing in the array has to start at zero: the latencies, the prefix state and the plan's lists are
    // written before they are read, and the progress word of the hand-over is cleared by the kernel that
    // sorts the plan.
    return best_neighbor_on(ctx, ctx->static_scratch, o_max_bound, base_order, n, moves, K, s, o, M, tel_out,
                            result_out, (hipStream_t)stream);
}

int kvsched_horizon_step(kvsched_ctx *ctx, int32_t *order, int32_t n, const int32_t *moves, int32_t K,
                         const int32_t *s, const int32_t *o, int64_t M, int64_t completed_in, int32_t complete_every,
                         int64_t *tel_out, int32_t *completion_out, int64_t *result_out, void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!order || !moves || !result_out || completed_in < 0 || complete_every < 1) return KVSCHED_EINVAL;
    if (K < 1 || K == INT32_MAX) return KVSCHED_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    // scratch: [K+1] latencies of best_neighbor | new order [n] | completion rounds [n] | one latency
    const size_t tel_bytes = neighbor_scratch_bytes(K, n, ctx->o_max_bound);  // best_neighbor's part
    const size_t row_bytes = align256(sizeof(int32_t) * (size_t)n);
    rc = ensure_scratch(ctx, tel_bytes + 2 * row_bytes + 256);
    if (rc != KVSCHED_OK) return rc;
    char *base = (char *)ctx->d_scratch;
    int32_t *new_order = (int32_t *)(base + tel_bytes);
    int32_t *comp = completion_out ? completion_out : (int32_t *)(base + tel_bytes + row_bytes);
    int64_t *tel1 = (int64_t *)(base + tel_bytes + 2 * row_bytes);
    // 1. best move of the window (result_out[0..2]).  When the positions before the window are placed once for
    //    all moves, their completion rounds are kept and the state behind them serves the chosen order too.
    rc = ensure_horizon(ctx, n);
    if (rc != KVSCHED_OK) return rc;
    const HorizonBuffers keep = horizon_buffers(ctx, n);
    int32_t prefix_len = 0;
    rc = best_neighbor_on(ctx, ctx->d_scratch, ctx->o_max_bound, order, n, moves, K, s, o, M, tel_out, result_out, st,
                          &keep, comp, &prefix_len);
    if (rc != KVSCHED_OK) {
        ctx->hz_len = 0;
        return rc;
    }
    // 2. take it
    rc = kvs_launch_apply_best_move(order, n, moves, result_out, new_order, st);
    if (rc != KVSCHED_OK) return rc;
    if (hipMemcpyAsync(order, new_order, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return KVSCHED_EHIP;
    // 3. the chosen timeline, 4. how far it gets
    const int32_t o_bound = ctx->o_max_bound > 0 ? ctx->o_max_bound
                                                 : (ctx->h_words[KVS_W_OMAX] < 1 ? 1 : ctx->h_words[KVS_W_OMAX]);
    SimParams p;
    p.src.orders = order;
    p.src.base = nullptr;
    p.src.moves = nullptr;
    p.C = 1;
    p.n = n;
    p.s = s;
    p.o = o;
    p.M = (int32_t)M;
    p.tel_out = tel1;
    p.completion_out = comp;
    p.completion_by_position = 0;
    p.d_words = ctx->d_words;
    p.o_bound = o_bound;
    if (prefix_len > 0) {  // (only with the register kernel) no move touches these positions: the new order shares them
        p.k_begin = prefix_len;
        p.state_in = keep.state;
    }
    rc = p.o_bound <= KVS_REG_MAX_O ? kvs_launch_simulate_reg(p, st)
                                    : kvs_launch_simulate(p, ring_slots_for(o_bound), st);
    if (rc != KVSCHED_OK) return rc;
    return kvs_launch_horizon_advance(order, comp, o, n, completed_in, complete_every, result_out + 3, st);
}

int kvsched_online(kvsched_ctx *ctx, int32_t B, const int32_t *streams, int32_t N, const int32_t *a,
                   const int32_t *s, const int32_t *o, int64_t M, int32_t backlog_cap, int32_t *completion_out,
                   int32_t out_len, int64_t *stats_out, void *stream)
{
    int rc = check_common(ctx, N, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!streams || !a || !completion_out || !stats_out || B < 1 || out_len < 1 || backlog_cap < 1)
        return KVSCHED_EINVAL;
    if (backlog_cap > KVSCHED_ONLINE_MAX_BACKLOG) return KVSCHED_ERANGE;
    hipStream_t st = (hipStream_t)stream;
    int32_t o_bound = 0;
    rc = scan_and_bound(ctx, s, o, N, M, st, &o_bound);
    if (rc != KVSCHED_OK) return rc;
    if (o_bound > KVSCHED_ONLINE_MAX_O) return KVSCHED_ERANGE;
    int32_t H = 64;  // ring of the running requests' future memory: a slot per round of the longest decode
    while (H < o_bound) H <<= 1;
    // More streams than run at once: those with most work go first (the order needs 2 B ints of scratch).
    int32_t *order_scratch = nullptr;
    if (B > kOnlineOrderMinStreams) {
        rc = ensure_scratch(ctx, 2 * sizeof(int32_t) * (size_t)B);
        if (rc != KVSCHED_OK) return rc;
        order_scratch = (int32_t *)ctx->d_scratch;
    }
    return kvs_launch_online(B, streams, N, a, s, o, (int32_t)M, backlog_cap, H, completion_out, out_len, stats_out,
                             order_scratch, ctx->d_words, st);
}

int kvsched_simulate_resume_positions(kvsched_ctx *ctx, int32_t C, int32_t *resume_pos_out, void *stream)
{
    if (!ctx || !resume_pos_out || C < 1) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    hipStream_t st = (hipStream_t)stream;
    if (ctx->resume_rows == 0) {  // the last call placed every row from its first position
        hipLaunchKernelGGL(kvs_fill_zero_i32, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, resume_pos_out, C);
        return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
    }
    if (C != ctx->resume_rows) return KVSCHED_EINVAL;
    const size_t list_bytes = align256(sizeof(int32_t) * (size_t)C);
    const int32_t *blocks = (const int32_t *)ctx->d_scratch;
    const int32_t *sorted = (const int32_t *)((const char *)ctx->d_scratch + list_bytes);
    return kvs_launch_resume_plan(sorted, C, ctx->resume_first, blocks, resume_pos_out, st);
}

int kvsched_simulate_stop_positions(kvsched_ctx *ctx, int32_t C, int32_t n, int32_t *stop_pos_out, void *stream)
{
    if (!ctx || !stop_pos_out || C < 1 || n < 1) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    if (ctx->rejoin_offset != 0 && C != ctx->resume_rows) return KVSCHED_EINVAL;
    const int32_t *rejoin =
        ctx->rejoin_offset != 0 ? (const int32_t *)((const char *)ctx->d_scratch + ctx->rejoin_offset) : nullptr;
    return kvs_launch_stop_positions(rejoin, C, n, stop_pos_out, (hipStream_t)stream);
}

int kvsched_neighbor_stop_positions(kvsched_ctx *ctx, int32_t K, int32_t n, int32_t *stop_pos_out, void *stream)
{
    if (!ctx || !stop_pos_out || K < 1 || n < 1) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    if (ctx->neighbor_stop_offset != 0 && K != ctx->neighbor_moves) return KVSCHED_EINVAL;
    const int32_t *rejoin = ctx->neighbor_stop_offset != 0
                                ? (const int32_t *)((const char *)ctx->d_scratch + ctx->neighbor_stop_offset)
                                : nullptr;
    return kvs_launch_stop_positions(rejoin, K, n, stop_pos_out, (hipStream_t)stream);
}

int kvsched_simulate_predicted(kvsched_ctx *ctx, const int32_t *orders, int32_t C, int32_t n, const int32_t *s,
                               const int32_t *o, const int32_t *est0, int32_t E, int64_t M, int64_t *tel_out,
                               int32_t *completion_out, int32_t *evictions_out, void *stream)
{
    int rc = check_common(ctx, n, s, o, M);
    if (rc != KVSCHED_OK) return rc;
    if (!orders || !est0 || !tel_out || C < 1 || (E != 1 && E != C)) return KVSCHED_EINVAL;
    if (n > 65535) return KVSCHED_ERANGE;
    hipStream_t st = (hipStream_t)stream;
    rc = kvs_launch_scan_lengths(s, o, n, (int32_t)M, ctx->o_max_bound, ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    int32_t bound = ctx->o_max_bound;
    if (bound <= 0) {
        rc = kvs_launch_scan_estimates(est0, (size_t)E * (size_t)n, ctx->d_words, st);
        if (rc != KVSCHED_OK) return rc;
        rc = read_words(ctx, st);
        if (rc != KVSCHED_OK) return rc;
        bound = ctx->h_words[KVS_W_OMAX] > ctx->h_words[KVS_W_ESTMAX] ? ctx->h_words[KVS_W_OMAX]
                                                                      : ctx->h_words[KVS_W_ESTMAX];
    }
    if (bound > KVSCHED_MAX_O) return KVSCHED_ERANGE;
    const int32_t H = ring_slots_for(bound < 1 ? 1 : bound);
    if (kvs_predicted_lds_bytes(n, H) > KVS_PREDICTED_MAX_LDS) return KVSCHED_ERANGE;
    // which candidates need the second launch; the estimates that stopped requests keep (written before read)
    const size_t retry_bytes = align256(sizeof(int32_t) * (size_t)C);
    rc = ensure_scratch(ctx, retry_bytes + sizeof(uint16_t) * (size_t)C * (size_t)n);
    if (rc != KVSCHED_OK) return rc;
    rc = kvs_launch_predicted(orders, C, n, s, o, est0, E, (int32_t)M, H, 1 << 26, tel_out, completion_out,
                              evictions_out, (int32_t *)ctx->d_scratch, (uint16_t *)((char *)ctx->d_scratch + retry_bytes),
                              ctx->d_words, st);
    if (rc != KVSCHED_OK) return rc;
    return kvs_launch_check_orders(orders, C, n, tel_out, ctx->d_words, st);
}

int kvsched_argmin(kvsched_ctx *ctx, const int64_t *tel, int32_t C, int64_t *result_out, void *stream)
{
    if (!ctx || !tel || !result_out || C < 1) return KVSCHED_EINVAL;
    if (hipSetDevice(ctx->device) != hipSuccess) return KVSCHED_EHIP;
    return kvs_launch_argmin(tel, C, result_out, 0, (hipStream_t)stream);
}

}  // extern "C"
