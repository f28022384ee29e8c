// Host side of the BUZZ decode library: C ABI, validation, workspace layout and the integer
// bookkeeping of Alg. 1 (sizes of sink / old / new / window regions).  Every size is a function of
// the configuration and the call history, so nothing is ever read back from the device.
#include <math.h>
#include <new>
#include <vector>

#include "buzz_internal.h"

using namespace buzz;

// Scratch of buzz_decode_step_static: the arrival counters and the per-split partial results of the split
// softmax, for callers that must not allocate.  One copy per GPU, held until the process ends; every call
// on a GPU shares it.  In host code this name is only a handle for hipGetSymbolAddress: the device address
// is looked up once per device and kept in g_static_scratch[].
constexpr size_t kStaticTicketBytes = 65536 * sizeof(int32_t);          // one counter per unit (units <= 65535)
constexpr size_t kStaticPartialBytes = (size_t)8 << 20;                 // (max, sum) pairs and partial outputs
constexpr size_t kStaticScratchBytes = kStaticTicketBytes + kStaticPartialBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices];   // device address of `scratch` on each GPU, nullptr until first use there

// Device address of this GPU's copy of the static scratch array (looked up once per device).
int static_scratch_ptr(char** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BUZZ_EHIP;
    if (!g_static_scratch[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BUZZ_EHIP;
        g_static_scratch[dev] = p;
    }
    *out = (char*)g_static_scratch[dev];
    return BUZZ_OK;
}

// Which die (XCD) a block runs on, for every block of a small 2-D grid: the evidence for placing a unit's
// splits on one die by block number (see die_local_ok).
__global__ void die_probe_kernel(int32_t* out)
{
    if (threadIdx.x == 0)
        out[blockIdx.y * gridDim.x + blockIdx.x] = (int32_t)(__builtin_amdgcn_s_getreg((31 << 11) | 20) & 7u);   // XCC_ID
}

int g_die_local[kMaxDevices];          // per GPU: 0 not probed yet, 1 blocks b and b + 8 share a die, 2 they do not
uint32_t g_die_map[kMaxDevices];       // per GPU: the die of block numbers 0..7, 4 bits each

// The die-local merge of the decode kernel relies on the hardware dealing the blocks of a grid to the dies
// round-robin in launch order (block b on die b mod 8), so that blocks whose numbers agree mod 8 share a die
// and its L2.  This checks that property once per GPU and process on two grid shapes, with one synchronisation
// of `st`; where it does not hold the decode step merges through device memory as it does for other shapes.
// Called from the prefill (never from a decode step, which must not synchronise).
int probe_die_placement(hipStream_t st)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BUZZ_EHIP;
    if (g_die_local[dev]) return BUZZ_OK;
    char* sp = nullptr;
    if (int rc = static_scratch_ptr(&sp)) return rc;
    int32_t* buf = (int32_t*)(sp + kStaticTicketBytes);                  // the partials area of the static scratch
    constexpr int kA = 8 * 64, kB = 3 * 40;
    int32_t host[kA + kB];
    hipLaunchKernelGGL(die_probe_kernel, dim3(8, 64), dim3(64), 0, st, buf);
    hipLaunchKernelGGL(die_probe_kernel, dim3(3, 40), dim3(64), 0, st, buf + kA);
    if (hipGetLastError() != hipSuccess) return BUZZ_EHIP;
    if (hipMemcpyAsync(host, buf, sizeof(host), hipMemcpyDeviceToHost, st) != hipSuccess) return BUZZ_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return BUZZ_EHIP;
    bool ok = true;
    for (int b = 8; b < kA; ++b) ok &= host[b] == host[b & 7];
    for (int b = 8; b < kB; ++b) ok &= host[kA + b] == host[kA + (b & 7)];
    uint32_t map = 0;
    for (int b = 0; b < 8; ++b) map |= (uint32_t)(host[b] & 7) << (4 * b);
    g_die_map[dev] = map;
    g_die_local[dev] = ok ? 1 : 2;
    return BUZZ_OK;
}

// Whether this GPU passed the placement probe; *map = the die of block numbers 0..7.
bool die_local_ok(uint32_t* map)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices || g_die_local[dev] != 1) return false;
    *map = g_die_map[dev];
    return true;
}

constexpr uint32_t kMagic = 0xB0220C4Eu;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

struct Layout {
    size_t K, V, score, pos, logit[2], stat[2], ticket, part_ml, part_o, sel, stK, stV, stScore, stPos, pscore, obs_stats, total;
    int32_t cap, old_cap, ring_cap, ring_base, s_cap, sel_stride, st_rows;
    int32_t units, G, elem, row_bytes, old_stride, keep;
};

int make_layout(const buzz_config_t* c, Layout* L)
{
    if (!c) return BUZZ_EINVAL;
    if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1) return BUZZ_EINVAL;
    if (c->n_q_heads % c->n_kv_heads) return BUZZ_EINVAL;
    if (c->kv_dtype < BUZZ_FP32 || c->kv_dtype > BUZZ_BF16) return BUZZ_EINVAL;
    if (c->sink < 0 || c->window < 0 || c->segment < 1 || c->keep < 0 || c->evict_every < 1) return BUZZ_EINVAL;
    if (c->old_stride < 0 || c->max_context < 1 || c->capacity < 0 || c->reserved != 0) return BUZZ_EINVAL;
    if (c->flags & ~(uint32_t)(BUZZ_FLAG_AUTO_EVICT | BUZZ_FLAG_DRY_RUN | BUZZ_FLAG_STREAMING | BUZZ_FLAG_CACHED |
                              BUZZ_FLAG_LOG_N | BUZZ_FLAG_THRESHOLD_TOTAL | BUZZ_FLAG_DETERMINISTIC |
                              BUZZ_FLAG_INTERVAL_NEW | BUZZ_FLAG_DEVICE_MERGE | BUZZ_FLAG_GLOBAL_TOPK))
        return BUZZ_EINVAL;
    if ((c->flags & BUZZ_FLAG_STREAMING) && (c->flags & BUZZ_FLAG_CACHED)) return BUZZ_EINVAL;
    if ((c->flags & BUZZ_FLAG_GLOBAL_TOPK) && (c->flags & (BUZZ_FLAG_THRESHOLD_TOTAL | BUZZ_FLAG_INTERVAL_NEW))) return BUZZ_EINVAL;
    if (!(c->softmax_scale >= 0.f) || isinf(c->softmax_scale)) return BUZZ_EINVAL;
    const int G = c->n_q_heads / c->n_kv_heads;
    if (!attn_supported(c->kv_dtype, c->head_dim, G)) return BUZZ_EUNSUPPORTED;
    if (c->segment > (1 << 28)) return BUZZ_EUNSUPPORTED;
    const int64_t units = (int64_t)c->batch * c->n_kv_heads;
    if (units > 65535) return BUZZ_EUNSUPPORTED;
    if (c->max_context > (1 << 28)) return BUZZ_EUNSUPPORTED;

    const int64_t k = c->sink, w = c->window, s = c->segment, T = c->evict_every;
    const bool global = c->flags & BUZZ_FLAG_GLOBAL_TOPK;       // one segment over everything between sink and window
    const int64_t keep = (global || c->keep < c->segment) ? c->keep : c->segment;   // a segment cannot yield more rows than it has
    const int64_t M = c->max_context > k + w ? c->max_context - k - w : 0;   // tokens that can ever be "new"
    int64_t old_cap;
    if (global) {
        old_cap = keep < M ? keep : M;                          // the survivors of the one segment
        if (c->capacity > 0 && c->capacity < k + old_cap + w + T) return BUZZ_EINVAL;
    } else if (c->capacity > 0) {
        old_cap = c->capacity - k - w - T;
        if (old_cap < 0) return BUZZ_EINVAL;
    } else if (c->flags & BUZZ_FLAG_THRESHOLD_TOTAL) {
        old_cap = keep == 0 ? 0 : T;                            // old + new never exceed T
    } else {
        const int64_t bound = keep * (ceil_div(M, s) + ceil_div(M, T) + 1);
        old_cap = keep == 0 ? 0 : (bound < M ? bound : M);
    }
    const int64_t ring = w + T;
    const int64_t cap = (int64_t)align_up((size_t)(k + old_cap + ring), 64);
    if (cap > (1 << 28)) return BUZZ_EUNSUPPORTED;

    L->units = (int32_t)units;
    L->G = G;
    L->elem = c->kv_dtype == BUZZ_FP32 ? 4 : 2;
    L->row_bytes = c->head_dim * L->elem;
    L->old_stride = c->old_stride > 0 ? c->old_stride : (c->segment + 1) / 2;
    L->keep = (int32_t)keep;
    L->cap = (int32_t)cap;
    L->old_cap = (int32_t)old_cap;
    L->ring_cap = (int32_t)ring;
    L->ring_base = (int32_t)(cap - ring);
    int64_t s_cap = kMaxBlocks / units;
    if (s_cap < 1) s_cap = 1;
    if (s_cap > kMaxSplits) s_cap = kMaxSplits;
    const int64_t s_need = ceil_div(cap * G, kStageFloats - 260 * G) + 1;   // a split's logits must fit the LDS staging
    if (s_need > kMaxSplits) return BUZZ_EUNSUPPORTED;
    if (s_cap < s_need) s_cap = s_need;
    L->s_cap = (int32_t)s_cap;
    const int64_t sel_bound = keep * (ceil_div(M, s) + 1);
    L->sel_stride = (int32_t)(keep == 0 ? 1 : (sel_bound < M ? sel_bound : (M > 0 ? M : 1)));
    L->st_rows = L->old_stride > 1 ? (int32_t)ceil_div(old_cap, L->old_stride) + 1 : 0;
    if (global) {                                               // survivors pass through the staging rows
        L->sel_stride = (int32_t)(old_cap > 0 ? old_cap : 1);
        L->st_rows = (int32_t)old_cap;
    }

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    const size_t rows = (size_t)units * cap;
    L->K = take(rows * L->row_bytes);
    L->V = take(rows * L->row_bytes);
    L->score = take(rows * 4);
    L->pos = take(rows * 4);
    L->logit[0] = take(rows * G * 4);
    L->logit[1] = take(rows * G * 4);
    L->stat[0] = take((size_t)units * G * 2 * 4);
    L->stat[1] = take((size_t)units * G * 2 * 4);
    L->ticket = take((size_t)units * 4);
    L->part_ml = take((size_t)units * s_cap * G * 2 * 4);
    L->part_o = take((size_t)units * s_cap * G * c->head_dim * 4);
    L->sel = take((size_t)units * L->sel_stride * 4);
    const size_t strows = (size_t)units * L->st_rows;
    L->stK = take(strows * L->row_bytes);
    L->stV = take(strows * L->row_bytes);
    L->stScore = take(strows * 4);
    L->stPos = take(strows * 4);
    L->pscore = take((size_t)units * c->max_context * 4);
    {   // prefill scoring statistics: what the vector path (fp32) or the matrix-core path (16-bit) needs
        const size_t vec = (size_t)units * ceil_div(c->max_context, kObsKeyBlock) * kObsRows * 2 * 4;
        const size_t mma = (size_t)c->batch * c->n_q_heads * kObsKeySplits * kObsPassRows * 2 * 4;
        L->obs_stats = take(c->kv_dtype == BUZZ_FP32 ? vec : mma);
    }
    L->total = off;
    return BUZZ_OK;
}

}  // namespace

struct buzz_cache {
    uint32_t magic;
    buzz_config_t cfg;
    Layout L;
    char* ws;
    float scale;
    bool dry;
    // state (Alg. 1): n = sink_filled + n_old + tail
    bool ready;
    int64_t sink_filled, n_old, tail, head, tokens_seen;
    int32_t user_splits;
    int64_t die_map_override;   // >= 0: use this instead of the placement probe's record (failure-handling tests)
    // the score update of the last decode step is applied lazily (by the next step or by a flush)
    bool pending;
    int last_buf;   // logit / stat buffer the last decode step wrote
    // benchmark profiling: event pairs per kernel class (0 attn, 1 epilogue, 2 eviction)
    bool prof;
    std::vector<hipEvent_t> ev[3];
    double prof_row_bytes;
    int64_t prof_evictions;

    int64_t n() const { return sink_filled + n_old + tail; }
    int64_t new_count() const
    {
        const int64_t v = n() - cfg.sink - n_old - cfg.window;
        return v > 0 ? v : 0;
    }
    int64_t trigger_count() const                               // what is compared with T
    {
        return (cfg.flags & BUZZ_FLAG_THRESHOLD_TOTAL) ? n_old + new_count() : new_count();
    }
    double log_n_factor(int64_t n_ctx) const                    // Sec. 3.5: log_512(n) for a query that sees n tokens
    {
        return (cfg.flags & BUZZ_FLAG_LOG_N) ? log((double)n_ctx) / log(512.0) : 1.0;
    }
    RingMap map() const
    {
        RingMap m;
        m.front = (int32_t)(sink_filled + n_old);
        m.ring_base = L.ring_base;
        m.ring_head = (int32_t)head;
        m.ring_cap = L.ring_cap;
        return m;
    }
    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

inline bool alive(const buzz_cache_t* c) { return c && c->magic == kMagic; }

// compute units of the current device (queried once, at the first launch)
int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cus = v;
        else
            cus = kDefaultCUs;
    }
    return cus;
}

constexpr size_t kMaxProfEvents = 1 << 15;

// a fresh event pair for one launch of kernel class `cls` while profiling is on, else an empty Timing
inline Timing prof_pair(buzz_cache_t* c, int cls)
{
    Timing tm;
    if (!c->prof || c->ev[cls].size() >= kMaxProfEvents) return tm;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return tm;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return tm; }
    c->ev[cls].push_back(a);
    c->ev[cls].push_back(b);
    tm.begin = a; tm.end = b;
    return tm;
}

void prof_clear(buzz_cache_t* c)
{
    for (auto& v : c->ev) {
        for (hipEvent_t e : v) (void)hipEventDestroy(e);
        v.clear();
    }
    c->prof_row_bytes = 0.0;
    c->prof_evictions = 0;
}
inline int hip_rc(hipError_t e) { return e == hipSuccess ? BUZZ_OK : BUZZ_EHIP; }

GatherArgs cache_gather_base(const buzz_cache_t* c)
{
    GatherArgs g{};
    g.srcK = c->at<char>(c->L.K); g.srcV = c->at<char>(c->L.V);
    g.srcScore = c->at<float>(c->L.score); g.srcPos = c->at<int32_t>(c->L.pos);
    g.src_unit_rows = c->L.cap;
    g.src_step = 1; g.sel_step = 1;
    g.dstK = c->at<char>(c->L.K); g.dstV = c->at<char>(c->L.V);
    g.dstScore = c->at<float>(c->L.score); g.dstPos = c->at<int32_t>(c->L.pos);
    g.dst_unit_rows = c->L.cap;
    g.row_bytes = c->L.row_bytes;
    return g;
}

// Sizes an eviction (the eviction branch of Alg. 1) would leave behind on a cache of n rows, n_old of them old:
// old2 interval-sampled old rows, new2 segment survivors out of newc new rows.  False when nothing would be
// evicted (Remark 1: no more than sink + window rows).
struct EvictSizes { int64_t newc, old2, new2; };
bool evict_sizes(const buzz_cache_t* c, int64_t n, int64_t n_old, EvictSizes* z)
{
    const int64_t k = c->cfg.sink, w = c->cfg.window, s = c->cfg.segment, keep = c->L.keep;
    if (n <= k + w) return false;
    const int64_t newc = n - k - n_old - w > 0 ? n - k - n_old - w : 0;
    z->newc = newc;
    if (c->cfg.flags & BUZZ_FLAG_GLOBAL_TOPK) {                // old and new rows are one segment
        z->old2 = 0;
        z->new2 = keep < n - k - w ? keep : n - k - w;
        return true;
    }
    z->old2 = ceil_div(n_old, c->L.old_stride);                // interval sampling keeps offsets 0, s^, 2 s^, ...
    z->new2 = keep * (newc / s) + (newc % s < keep ? newc % s : keep);   // every segment yields min(keep, len)
    return true;
}

// Whether an eviction with these sizes stays inside what the workspace layout set aside: the old region
// (which ends where the ring begins), the list of selected rows, the staging rows.  The old-region bound is
// the caller-visible capacity; the others hold by construction of the layout and are checked all the same,
// before anything is enqueued: a launch must never be given a row the workspace does not have.
bool evict_uses_one_launch(const buzz_cache_t* c, int64_t n_old, const EvictSizes& z)
{
    return !(c->cfg.flags & BUZZ_FLAG_GLOBAL_TOPK) && z.old2 == n_old &&
           ((int64_t)c->cfg.segment + c->L.keep) * (int64_t)(4 * sizeof(float)) <= 65536;
}
bool evict_fits(const buzz_cache_t* c, int64_t n_old, const EvictSizes& z)
{
    const Layout& L = c->L;
    if (z.old2 + z.new2 > L.old_cap) return false;
    if (c->cfg.sink + z.old2 + z.new2 > L.ring_base) return false;
    if (c->cfg.flags & BUZZ_FLAG_GLOBAL_TOPK) return z.new2 <= L.st_rows && z.new2 <= L.sel_stride;
    if (evict_uses_one_launch(c, n_old, z)) return true;
    if (z.old2 < n_old && z.old2 > L.st_rows) return false;
    return z.new2 <= L.sel_stride;
}

// Applies the score update the last decode step left pending, so that the scores are current.
int flush_scores(buzz_cache_t* c, hipStream_t st)
{
    if (!c->pending || c->dry) { c->pending = false; return BUZZ_OK; }
    const Layout& L = c->L;
    AttnArgs a{};
    a.score = c->at<float>(L.score);
    a.logit_prev = c->at<float>(L.logit[c->last_buf]);
    a.stat_prev = c->at<float>(L.stat[c->last_buf]);
    a.map = c->map();
    a.n = (int32_t)c->n();
    a.cap = L.cap;
    if (hipError_t e = launch_flush_scores(L.G, a, L.units, st, prof_pair(c, 1))) return hip_rc(e);
    c->pending = false;
    return BUZZ_OK;
}

// The eviction branch of Alg. 1 on the current state.
int evict_impl(buzz_cache_t* c, hipStream_t st)
{
    const buzz_config_t& cfg = c->cfg;
    const Layout& L = c->L;
    const int64_t k = cfg.sink;
    EvictSizes z;
    if (!evict_sizes(c, c->n(), c->n_old, &z)) return BUZZ_OK; // Remark 1
    const int64_t newc = z.newc, sh = L.old_stride, old2 = z.old2, new2 = z.new2;
    if (!evict_fits(c, c->n_old, z)) return BUZZ_ECAPACITY;
    if (cfg.flags & BUZZ_FLAG_GLOBAL_TOPK) {
        // H2O-style: the top `keep` of ALL rows between sink and window survive.  Survivors may sit anywhere in
        // the old region or the ring and land where old rows are, so they travel through the staging rows.
        if (int rc = flush_scores(c, st)) return rc;
        if (!c->dry && new2 > 0) {
            if (c->prof) c->prof_evictions += 1;
            const int64_t mid = c->n() - k - cfg.window;
            SelectArgs sa{};
            sa.score = c->at<float>(L.score); sa.unit_stride = L.cap;
            sa.map = c->map(); sa.lo = (int32_t)k; sa.new_count = (int32_t)mid;
            sa.segment = (int32_t)(mid > kMaxWaveSegment ? mid : kMaxWaveSegment);   // one segment, whatever its length
            sa.keep = L.keep; sa.ignore_scores = 0;
            sa.sel = c->at<int32_t>(L.sel); sa.sel_stride = L.sel_stride;
            if (hipError_t e = launch_segment_topk(sa, L.units, st, prof_pair(c, 2))) return hip_rc(e);
            GatherArgs g = cache_gather_base(c);
            g.src_map = c->map();
            g.sel = c->at<int32_t>(L.sel); g.sel_stride = L.sel_stride; g.sel_start = 0; g.sel_step = 1;
            g.dstK = c->at<char>(L.stK); g.dstV = c->at<char>(L.stV);
            g.dstScore = c->at<float>(L.stScore); g.dstPos = c->at<int32_t>(L.stPos);
            g.dst_unit_rows = L.st_rows; g.dst_start = 0; g.n_rows = (int32_t)new2;
            if (hipError_t e = launch_gather_rows(g, L.units, st, prof_pair(c, 2))) return hip_rc(e);
            GatherArgs b = cache_gather_base(c);
            b.srcK = c->at<char>(L.stK); b.srcV = c->at<char>(L.stV);
            b.srcScore = c->at<float>(L.stScore); b.srcPos = c->at<int32_t>(L.stPos);
            b.src_unit_rows = L.st_rows; b.src_start = 0; b.src_step = 1;
            b.dst_start = (int32_t)k; b.n_rows = (int32_t)new2;
            if (hipError_t e = launch_gather_rows(b, L.units, st, prof_pair(c, 2))) return hip_rc(e);
        }
        c->n_old = new2;
        c->head = (c->head + newc) % L.ring_cap;
        c->tail -= newc;
        return BUZZ_OK;
    }
    // Old rows that stay where they are (old stride 1) leave only the new rows to deal with, and one launch
    // does that: a score update still pending stays pending for every row that keeps its place.
    const bool in_place = evict_uses_one_launch(c, c->n_old, z);
    if (in_place) {
        if (!c->dry && new2 > 0) {
            if (c->prof) c->prof_evictions += 1;
            EvictArgs ea{};
            ea.K = c->at<char>(L.K); ea.V = c->at<char>(L.V);
            ea.score = c->at<float>(L.score); ea.pos = c->at<int32_t>(L.pos);
            ea.logit_prev = c->pending ? c->at<float>(L.logit[c->last_buf]) : nullptr;
            ea.stat_prev = c->at<float>(L.stat[c->last_buf]);
            ea.map = c->map(); ea.lo = ea.map.front; ea.new_count = (int32_t)newc;
            ea.segment = cfg.segment; ea.keep = L.keep;
            ea.ignore_scores = (cfg.flags & BUZZ_FLAG_INTERVAL_NEW) ? 1 : 0;
            ea.dst_start = (int32_t)(k + old2);
            ea.cap = L.cap; ea.row_bytes = L.row_bytes; ea.G = L.G;
            if (hipError_t e = launch_evict_new_rows(ea, L.units, st, prof_pair(c, 2))) return hip_rc(e);
        } else if (!c->dry && c->prof) {
            c->prof_evictions += 1;
        }
        c->n_old = old2 + new2;
        c->head = (c->head + newc) % L.ring_cap;
        c->tail -= newc;
        return BUZZ_OK;
    }
    if (int rc = flush_scores(c, st)) return rc;              // the selection reads the scores
    if (!c->dry) {
        if (c->prof) c->prof_evictions += 1;
        if (old2 < c->n_old) {                                 // thin the old region through the staging rows
            GatherArgs g = cache_gather_base(c);
            g.src_start = (int32_t)k; g.src_step = (int32_t)sh;
            g.dstK = c->at<char>(L.stK); g.dstV = c->at<char>(L.stV);
            g.dstScore = c->at<float>(L.stScore); g.dstPos = c->at<int32_t>(L.stPos);
            g.dst_unit_rows = L.st_rows; g.dst_start = 0; g.n_rows = (int32_t)old2;
            if (hipError_t e = launch_gather_rows(g, L.units, st, prof_pair(c, 2))) return hip_rc(e);
            GatherArgs b = cache_gather_base(c);
            b.srcK = c->at<char>(L.stK); b.srcV = c->at<char>(L.stV);
            b.srcScore = c->at<float>(L.stScore); b.srcPos = c->at<int32_t>(L.stPos);
            b.src_unit_rows = L.st_rows; b.src_start = 0; b.src_step = 1;
            b.dst_start = (int32_t)k; b.n_rows = (int32_t)old2;
            if (hipError_t e = launch_gather_rows(b, L.units, st, prof_pair(c, 2))) return hip_rc(e);
        }
        if (new2 > 0) {
            SelectArgs sa{};
            sa.score = c->at<float>(L.score); sa.unit_stride = L.cap;
            sa.map = c->map(); sa.lo = sa.map.front; sa.new_count = (int32_t)newc;
            sa.segment = cfg.segment; sa.keep = L.keep;
            sa.ignore_scores = (cfg.flags & BUZZ_FLAG_INTERVAL_NEW) ? 1 : 0;
            sa.sel = c->at<int32_t>(L.sel); sa.sel_stride = L.sel_stride;
            if (hipError_t e = launch_segment_topk(sa, L.units, st, prof_pair(c, 2))) return hip_rc(e);
            GatherArgs g = cache_gather_base(c);
            g.src_map = c->map();
            g.sel = c->at<int32_t>(L.sel); g.sel_stride = L.sel_stride; g.sel_start = 0; g.sel_step = 1;
            g.dst_start = (int32_t)(k + old2); g.n_rows = (int32_t)new2;
            if (hipError_t e = launch_gather_rows(g, L.units, st, prof_pair(c, 2))) return hip_rc(e);
        }
    }
    c->n_old = old2 + new2;
    c->head = (c->head + newc) % L.ring_cap;
    c->tail -= newc;
    return BUZZ_OK;
}

}  // namespace

extern "C" {

int buzz_workspace_bytes(const buzz_config_t* cfg, size_t* bytes)
{
    if (!cfg || !bytes) return BUZZ_EINVAL;
    Layout L;
    if (int rc = make_layout(cfg, &L)) return rc;
    *bytes = L.total;
    return BUZZ_OK;
}

int buzz_cache_create(const buzz_config_t* cfg, void* dev_workspace, size_t bytes, buzz_cache_t** out)
{
    if (!cfg || !out) return BUZZ_EINVAL;
    Layout L;
    if (int rc = make_layout(cfg, &L)) return rc;
    const bool dry = cfg->flags & BUZZ_FLAG_DRY_RUN;
    if (!dry) {
        if (!dev_workspace || ((uintptr_t)dev_workspace & 255)) return BUZZ_EINVAL;
        if (bytes < L.total) return BUZZ_ECAPACITY;
    }
    buzz_cache_t* c = new (std::nothrow) buzz_cache_t();
    if (!c) return BUZZ_EINVAL;
    c->magic = kMagic;
    c->cfg = *cfg;
    c->L = L;
    c->ws = (char*)dev_workspace;
    c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
    c->dry = dry;
    c->ready = false;
    c->sink_filled = c->n_old = c->tail = c->head = c->tokens_seen = 0;
    c->user_splits = 0;
    c->die_map_override = -1;
    c->pending = false;
    c->last_buf = 0;
    c->prof = false;
    c->prof_row_bytes = 0.0;
    c->prof_evictions = 0;
    *out = c;
    return BUZZ_OK;
}

int buzz_cache_destroy(buzz_cache_t* c)
{
    if (!c) return BUZZ_OK;
    if (!alive(c)) return BUZZ_EINVAL;
    prof_clear(c);
    c->magic = 0;
    delete c;
    return BUZZ_OK;
}

int buzz_cache_len(const buzz_cache_t* c, int64_t* n, int64_t* n_old, int64_t* new_count)
{
    if (!alive(c)) return BUZZ_EINVAL;
    if (n) *n = c->n();
    if (n_old) *n_old = c->n_old;
    if (new_count) *new_count = c->new_count();
    return BUZZ_OK;
}

int buzz_cache_set_splits(buzz_cache_t* c, int32_t n_splits)
{
    if (!alive(c) || n_splits < 0 || n_splits > c->L.s_cap) return BUZZ_EINVAL;
    c->user_splits = n_splits;
    return BUZZ_OK;
}

int buzz_cache_override_die_map(buzz_cache_t* c, int64_t die_map)
{
    if (!alive(c) || die_map > 0xffffffffll) return BUZZ_EINVAL;
    c->die_map_override = die_map < 0 ? -1 : die_map;
    return BUZZ_OK;
}

int buzz_prefill(buzz_cache_t* c, const void* kp, const void* vp, int64_t N, const void* q_obs, int64_t n_obs,
                 const float* init_score, void* hip_stream)
{
    if (!alive(c)) return BUZZ_EINVAL;
    if (N < 0 || n_obs < 0 || n_obs > N) return BUZZ_EINVAL;
    if (N > 0 && !c->dry && (!kp || !vp)) return BUZZ_EINVAL;
    if ((n_obs > 0) != (q_obs != nullptr) && !c->dry) return BUZZ_EINVAL;
    const buzz_config_t& cfg = c->cfg;
    const Layout& L = c->L;
    if (N > cfg.max_context) return BUZZ_ECAPACITY;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t k = cfg.sink, w = cfg.window, s = cfg.segment, keep = L.keep, T = cfg.evict_every;
    const int64_t M = N - k - w;                                // prompt tokens between sink and window
    const bool sample = M >= T;
    int64_t survivors = 0, selected = 0, sel_step = 1;
    const bool global = cfg.flags & BUZZ_FLAG_GLOBAL_TOPK;
    if (sample && global) {
        survivors = selected = keep < M ? keep : M;             // H2O-style: one segment over the whole middle
    } else if (sample) {
        const int64_t last = M % s < keep ? M % s : keep;
        survivors = selected = keep * (M / s) + last;           // rows the selection lists; Remark 2 may thin them
        if (L.old_stride > 1 && (cfg.capacity > 0 || (cfg.flags & BUZZ_FLAG_THRESHOLD_TOTAL))) {   // Remark 2: sample until it fits
            while (survivors > L.old_cap) {
                const int64_t nxt = ceil_div(survivors, L.old_stride);
                if (nxt >= survivors) return BUZZ_ECAPACITY;
                survivors = nxt;
                sel_step *= L.old_stride;
            }
        }
        if (survivors > L.old_cap) return BUZZ_ECAPACITY;
    }
    const int64_t sink_rows = N < k ? N : k;
    const int64_t tail_rows = sample ? w : N - sink_rows;
    if (tail_rows > L.ring_cap) return BUZZ_ECAPACITY;
    // the layout's own regions: selected rows fit the selection list, survivors end before the ring begins
    if (selected > L.sel_stride || sink_rows + survivors > L.ring_base) return BUZZ_ECAPACITY;

    if (!c->dry) {
        float* ps = c->at<float>(L.pscore);
        if (int rc = probe_die_placement(st)) return rc;
        if (hipError_t e = launch_fill_f32(c->at<float>(L.ticket), nullptr, L.units, st)) return hip_rc(e);
        // starting scores, one row of N per unit
        if (hipError_t e = launch_fill_f32(ps, init_score, (int64_t)L.units * N, st)) return hip_rc(e);
        if (n_obs > 0) {
            const int G = L.G;
            const int max_q = obs_pass_queries(cfg.kv_dtype, G);   // queries of one head per pass
            for (int64_t t0 = 0; t0 < n_obs; t0 += max_q) {
                ObsArgs oa{};
                oa.K = kp; oa.q_obs = q_obs; oa.score = ps; oa.stats = c->at<float>(L.obs_stats);
                oa.N = (int32_t)N; oa.n_obs = (int32_t)n_obs;
                oa.t_begin = (int32_t)t0; oa.t_count = (int32_t)((n_obs - t0) < max_q ? (n_obs - t0) : max_q);
                oa.Hq = cfg.n_q_heads; oa.Hkv = cfg.n_kv_heads;
                oa.scale_log2 = c->scale * 1.4426950408889634f;
                oa.log_n = (cfg.flags & BUZZ_FLAG_LOG_N) ? 1 : 0;
                {   // few observed queries leave the row-statistics step with fewer blocks than compute units:
                    // then up to kObsKeySplits blocks share a query group's keys (at least 512 keys each)
                    const int64_t blocks = (int64_t)cfg.batch * cfg.n_q_heads * ceil_div(oa.t_count, 256);
                    int64_t ks = ceil_div(3 * (int64_t)compute_units(), blocks);
                    if (ks > N / 512) ks = N / 512;
                    oa.key_splits = (int32_t)(ks < 1 ? 1 : (ks > kObsKeySplits ? kObsKeySplits : ks));
                }
                if (hipError_t e = launch_obs_scores(cfg.kv_dtype, cfg.head_dim, G, oa, L.units, st)) return hip_rc(e);
            }
        }
        GatherArgs g{};
        g.srcK = kp; g.srcV = vp; g.srcScore = ps; g.srcPos = nullptr;
        g.src_unit_rows = N; g.src_step = 1; g.sel_step = 1;
        g.dstK = c->at<char>(L.K); g.dstV = c->at<char>(L.V);
        g.dstScore = c->at<float>(L.score); g.dstPos = c->at<int32_t>(L.pos);
        g.dst_unit_rows = L.cap; g.row_bytes = L.row_bytes;
        // sink
        GatherArgs gs = g;
        gs.src_start = 0; gs.dst_start = 0; gs.n_rows = (int32_t)sink_rows;
        if (hipError_t e = launch_gather_rows(gs, L.units, st)) return hip_rc(e);
        if (sample) {
            if (survivors > 0) {
                SelectArgs sa{};
                sa.score = ps; sa.unit_stride = N;
                sa.map = RingMap{0, 0, 0, 0};
                sa.lo = (int32_t)k; sa.new_count = (int32_t)M;
                sa.segment = global ? (int32_t)(M > kMaxWaveSegment ? M : kMaxWaveSegment) : cfg.segment;
                sa.keep = L.keep;
                sa.ignore_scores = (cfg.flags & BUZZ_FLAG_INTERVAL_NEW) ? 1 : 0;
                sa.sel = c->at<int32_t>(L.sel); sa.sel_stride = L.sel_stride;
                if (hipError_t e = launch_segment_topk(sa, L.units, st)) return hip_rc(e);
                GatherArgs gv = g;
                gv.sel = c->at<int32_t>(L.sel); gv.sel_stride = L.sel_stride; gv.sel_start = 0;
                gv.sel_step = (int32_t)sel_step;
                gv.dst_start = (int32_t)k; gv.n_rows = (int32_t)survivors;
                if (hipError_t e = launch_gather_rows(gv, L.units, st)) return hip_rc(e);
            }
            GatherArgs gw = g;
            gw.src_start = (int32_t)(N - w); gw.dst_start = L.ring_base; gw.n_rows = (int32_t)w;
            if (hipError_t e = launch_gather_rows(gw, L.units, st)) return hip_rc(e);
        } else {
            GatherArgs gt = g;
            gt.src_start = (int32_t)sink_rows; gt.dst_start = L.ring_base; gt.n_rows = (int32_t)tail_rows;
            if (hipError_t e = launch_gather_rows(gt, L.units, st)) return hip_rc(e);
        }
    }
    c->pending = false;
    c->sink_filled = sink_rows;
    c->n_old = survivors;
    c->tail = tail_rows;
    c->head = 0;
    c->tokens_seen = N;
    c->ready = true;
    return BUZZ_OK;
}

}  // extern "C"

namespace {

// One decode step.  static_scratch: the split-softmax scratch (arrival counters, per-split partials) is the
// library's static device array instead of the caller's workspace.
int decode_step_impl(buzz_cache_t* c, const void* q, const void* k_new, const void* v_new, float* out,
                     void* hip_stream, bool static_scratch)
{
    if (!alive(c)) return BUZZ_EINVAL;
    if (!c->dry && (!q || !k_new || !v_new || !out)) return BUZZ_EINVAL;
    if (!c->ready) return BUZZ_ESTATE;
    if (static_scratch && c->prof) return BUZZ_ESTATE;         // the profiling pass creates events per launch
    const buzz_config_t& cfg = c->cfg;
    const Layout& L = c->L;
    if (c->tokens_seen >= cfg.max_context) return BUZZ_ECAPACITY;
    hipStream_t st = (hipStream_t)hip_stream;

    const bool to_sink = c->sink_filled < cfg.sink && c->n_old == 0 && c->tail == 0;   // Remark 1: sink first
    if (!to_sink && c->tail >= L.ring_cap) return BUZZ_ECAPACITY;
    const int64_t new_phys = to_sink ? c->sink_filled : L.ring_base + (c->head + c->tail) % L.ring_cap;
    // state after the append of eq. 2
    const int64_t sink_filled = c->sink_filled + (to_sink ? 1 : 0);
    const int64_t tail = c->tail + (to_sink ? 0 : 1);
    const int64_t n = sink_filled + c->n_old + tail;
    // With automatic eviction the step ends with one when the threshold is reached: whether its survivors fit
    // is known now, before anything is enqueued or changed.
    bool evict_after = false;
    if (cfg.flags & BUZZ_FLAG_AUTO_EVICT) {
        EvictSizes z;
        if (evict_sizes(c, n, c->n_old, &z)) {
            const int64_t count = (cfg.flags & BUZZ_FLAG_THRESHOLD_TOTAL) ? c->n_old + z.newc : z.newc;
            evict_after = count >= cfg.evict_every;
            if (evict_after && !evict_fits(c, c->n_old, z)) return BUZZ_ECAPACITY;
        }
    }

    // the row being written must lie inside the sink or the ring, the rows stored linearly before the ring
    if (to_sink ? (new_phys < 0 || new_phys >= cfg.sink)
                : (new_phys < L.ring_base || new_phys >= (int64_t)L.ring_base + L.ring_cap || new_phys >= L.cap))
        return BUZZ_ECAPACITY;
    if (sink_filled + c->n_old > L.ring_base) return BUZZ_ECAPACITY;
    // Key-range splits.  Few, long blocks amortise the per-block merge, and a block count that fills every
    // compute unit the same number of times avoids a tail.  Automatic choice: one block per compute unit, 8
    // waves wide (floor(CUs / units) splits); with at least one unit per CU a unit is a single block and nothing
    // is merged across blocks at all.
    const int cus = compute_units();
    const int tile = attn_tile_rows(cfg.kv_dtype, cfg.head_dim, L.G);
    int64_t S = c->user_splits > 0 ? c->user_splits : (L.units >= cus ? 1 : cus / L.units);
    // a split of fewer than kMinSplitRows rows costs more in merge latency than it saves in streaming
    if (c->user_splits == 0 && S > ceil_div(n, kMinSplitRows)) S = ceil_div(n, kMinSplitRows);
    if (S < 1) S = 1;
    if (S > L.s_cap) S = L.s_cap;
    int64_t rps = ceil_div(ceil_div(n, S), tile) * tile;
    const int stage_cap = stage_floats(L.G, cfg.head_dim);
    while ((rps + 4) * L.G > stage_cap) {                      // LDS staging bound (+ alignment slack)
        S += 1;
        rps = ceil_div(ceil_div(n, S), tile) * tile;
    }
    const int64_t n_splits = ceil_div(n, rps);
    // the workspace holds s_cap partial results per unit (the static scratch has its own bound below)
    if (!static_scratch && n_splits > L.s_cap) return BUZZ_ECAPACITY;

    if (!c->dry) {
        AttnArgs a{};
        a.q = q; a.k_new = k_new; a.v_new = v_new;
        a.K = c->at<char>(L.K); a.V = c->at<char>(L.V);
        a.score = c->at<float>(L.score); a.pos = c->at<int32_t>(L.pos);
        const int cur = c->last_buf ^ 1;
        a.logit = c->at<float>(L.logit[cur]); a.logit_prev = c->at<float>(L.logit[c->last_buf]);
        a.stat = c->at<float>(L.stat[cur]); a.stat_prev = c->at<float>(L.stat[c->last_buf]);
        a.ticket = c->at<int32_t>(L.ticket);
        a.pending = c->pending ? 1 : 0;
        a.part_ml = c->at<float>(L.part_ml); a.part_o = c->at<float>(L.part_o);
        a.out = out;
        a.map = c->map();
        a.map.front = (int32_t)(sink_filled + c->n_old);
        a.n = (int32_t)n;
        a.new_phys = (int32_t)new_phys;
        a.new_pos = (int32_t)c->tokens_seen;
        a.cap = L.cap;
        a.Hq = cfg.n_q_heads; a.Hkv = cfg.n_kv_heads;
        a.s_cap = L.s_cap;
        a.scale_log2 = (float)(c->scale * 1.4426950408889634 * c->log_n_factor(c->tokens_seen + 1));
        const double step_bytes = (double)L.units * (double)n * 2.0 * L.row_bytes;
        a.streaming = (cfg.flags & BUZZ_FLAG_STREAMING) ? 1
                      : (cfg.flags & BUZZ_FLAG_CACHED) ? 0 : (step_bytes > kLastLevelCacheBytes);
        a.fixed_tiles = (cfg.flags & BUZZ_FLAG_DETERMINISTIC) ? 1 : 0;
        a.rows_per_split = (int32_t)rps;
        a.n_splits = (int32_t)n_splits;
        if (static_scratch && a.n_splits > 1) {
            // partials are laid out [units][n_splits] in the static array; the counters are cleared by a small
            // kernel (not a memset: the caller may be capturing a graph), whatever the last call left there
            const size_t ml_bytes = align_up((size_t)L.units * a.n_splits * L.G * 2 * sizeof(float), 256);
            const size_t o_bytes = (size_t)L.units * a.n_splits * L.G * cfg.head_dim * sizeof(float);
            if (ml_bytes + o_bytes > kStaticPartialBytes) return BUZZ_ECAPACITY;
            char* sp = nullptr;
            if (int rc = static_scratch_ptr(&sp)) return rc;
            a.ticket = (int32_t*)sp;
            a.part_ml = (float*)(sp + kStaticTicketBytes);
            a.part_o = (float*)(sp + kStaticTicketBytes + ml_bytes);
            a.s_cap = a.n_splits;
            if (hipError_t e = launch_fill_f32((float*)sp, nullptr, L.units, st)) return hip_rc(e);
        }
        // about 8 waves per compute unit; 4-wave blocks also where 8 waves' partial outputs would not fit the LDS
        a.waves = ((int64_t)L.units * a.n_splits <= cus && L.G * cfg.head_dim < kWideBlockMaxGD) ? 8 : 4;
        // a unit's splits on one die, merged through that die's L2: possible when the units divide evenly over
        // the 8 dies
        a.xcd_local = (a.n_splits > 1 && L.units % 8 == 0 && !(cfg.flags & BUZZ_FLAG_DEVICE_MERGE) &&
                       die_local_ok(&a.die_map)) ? 1 : 0;
        if (a.xcd_local && c->die_map_override >= 0) a.die_map = (uint32_t)c->die_map_override;
        if (hipError_t e = launch_attn_split(cfg.kv_dtype, cfg.head_dim, L.G, a, L.units, st,
                                             static_scratch ? Timing{} : prof_pair(c, 0)))
            return hip_rc(e);
        if (c->prof) c->prof_row_bytes += (double)L.units * (double)n * 2.0 * L.row_bytes;
        c->last_buf = cur;
    }
    c->pending = true;
    c->sink_filled = sink_filled;
    c->tail = tail;
    c->tokens_seen += 1;
    if (evict_after || ((cfg.flags & BUZZ_FLAG_AUTO_EVICT) && c->trigger_count() >= cfg.evict_every))
        return evict_impl(c, st);                              // cannot fail for capacity: checked above
    return BUZZ_OK;
}

}  // namespace

extern "C" {

int buzz_decode_step(buzz_cache_t* c, const void* q, const void* k_new, const void* v_new, float* out,
                     void* hip_stream)
{
    return decode_step_impl(c, q, k_new, v_new, out, hip_stream, false);
}

int buzz_decode_step_static(buzz_cache_t* c, const void* q, const void* k_new, const void* v_new, float* out,
                            void* hip_stream)
{
    return decode_step_impl(c, q, k_new, v_new, out, hip_stream, true);
}

int buzz_evict(buzz_cache_t* c, void* hip_stream)
{
    if (!alive(c)) return BUZZ_EINVAL;
    if (!c->ready) return BUZZ_ESTATE;
    return evict_impl(c, (hipStream_t)hip_stream);
}

int buzz_cache_export(buzz_cache_t* c, void* k, void* v, float* score, int32_t* pos, void* hip_stream)
{
    if (!alive(c)) return BUZZ_EINVAL;
    if (!c->ready) return BUZZ_ESTATE;
    if (c->dry) return BUZZ_OK;
    if (int rc = flush_scores(c, (hipStream_t)hip_stream)) return rc;
    GatherArgs g = cache_gather_base(c);
    g.src_map = c->map();
    g.src_start = 0; g.src_step = 1;
    g.dstK = k; g.dstV = v; g.dstScore = score; g.dstPos = pos;
    g.dst_unit_rows = c->n(); g.dst_start = 0; g.n_rows = (int32_t)c->n();
    return hip_rc(launch_gather_rows(g, c->L.units, (hipStream_t)hip_stream));
}

int buzz_cache_import(buzz_cache_t* c, const void* k, const void* v, const float* score, const int32_t* pos,
                      int64_t n, int64_t n_old, int64_t tokens_seen, void* hip_stream)
{
    if (!alive(c) || n < 0 || n_old < 0 || n_old > n || tokens_seen < n) return BUZZ_EINVAL;
    if (!c->dry && n > 0 && (!k || !v || !score || !pos)) return BUZZ_EINVAL;
    const buzz_config_t& cfg = c->cfg;
    const Layout& L = c->L;
    if (tokens_seen > cfg.max_context || n_old > L.old_cap) return BUZZ_ECAPACITY;
    // Alg. 1 fills the sink first, and old rows only exist once the sink is full
    const int64_t sink_rows = n - n_old < cfg.sink ? n - n_old : cfg.sink;
    if (n_old > 0 && sink_rows < cfg.sink) return BUZZ_EINVAL;
    const int64_t tail_rows = n - sink_rows - n_old;
    if (tail_rows > L.ring_cap || sink_rows + n_old > L.ring_base) return BUZZ_ECAPACITY;
    if (!c->dry) {
        hipStream_t st = (hipStream_t)hip_stream;
        if (int rc = probe_die_placement(st)) return rc;
        if (hipError_t e = launch_fill_f32(c->at<float>(L.ticket), nullptr, L.units, st)) return hip_rc(e);
        GatherArgs g{};
        g.srcK = k; g.srcV = v; g.srcScore = score; g.srcPos = pos;
        g.src_unit_rows = n; g.src_step = 1; g.sel_step = 1;
        g.dstK = c->at<char>(L.K); g.dstV = c->at<char>(L.V);
        g.dstScore = c->at<float>(L.score); g.dstPos = c->at<int32_t>(L.pos);
        g.dst_unit_rows = L.cap; g.row_bytes = L.row_bytes;
        GatherArgs front = g;                                  // sink and old rows: the linear region
        front.src_start = 0; front.dst_start = 0; front.n_rows = (int32_t)(sink_rows + n_old);
        if (hipError_t e = launch_gather_rows(front, L.units, st)) return hip_rc(e);
        GatherArgs ring = g;                                   // buffered new rows and the window: the ring, from its base
        ring.src_start = (int32_t)(sink_rows + n_old); ring.dst_start = L.ring_base; ring.n_rows = (int32_t)tail_rows;
        if (hipError_t e = launch_gather_rows(ring, L.units, st)) return hip_rc(e);
    }
    c->pending = false;
    c->sink_filled = sink_rows;
    c->n_old = n_old;
    c->tail = tail_rows;
    c->head = 0;
    c->tokens_seen = tokens_seen;
    c->ready = true;
    return BUZZ_OK;
}

int buzz_cache_profile(buzz_cache_t* c, int enable)
{
    if (!alive(c)) return BUZZ_EINVAL;
    if (enable) prof_clear(c);
    c->prof = enable != 0 && !c->dry;
    return BUZZ_OK;
}

int buzz_cache_profile_read(buzz_cache_t* c, buzz_profile_t* out)
{
    if (!alive(c) || !out) return BUZZ_EINVAL;
    double ms[3] = {0, 0, 0};
    int64_t cnt[3] = {0, 0, 0};
    for (int cls = 0; cls < 3; ++cls) {
        const auto& v = c->ev[cls];
        for (size_t i = 0; i + 1 < v.size(); i += 2) {
            if (hipEventSynchronize(v[i + 1]) != hipSuccess) return BUZZ_EHIP;
            float t = 0.f;
            if (hipEventElapsedTime(&t, v[i], v[i + 1]) != hipSuccess) return BUZZ_EHIP;
            ms[cls] += t;
            cnt[cls] += 1;
        }
    }
    out->attn_launches = cnt[0]; out->epilogue_launches = cnt[1]; out->evictions = c->prof_evictions;
    out->attn_ms = ms[0]; out->epilogue_ms = ms[1]; out->evict_ms = ms[2];
    out->attn_row_bytes = c->prof_row_bytes;
    return BUZZ_OK;
}

int buzz_bench_copy(void* dst, const void* src, size_t bytes, void* hip_stream)
{
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return BUZZ_EINVAL;
    return hip_rc(launch_plain_copy(dst, src, bytes, (hipStream_t)hip_stream));
}

int64_t buzz_suggest_threshold(int32_t segment, int32_t window)
{
    if (segment < 1 || window < 0) return 0;
    const double s = segment, w = window;
    const double t = (segment & 1) ? w * (s * s + 1.0) / (s + 1.0) : w * (s - 1.0);
    const int64_t r = (int64_t)floor(t + 0.5);
    return r < 1 ? 1 : r;
}

const char* buzz_strerror(int status)
{
    switch (status) {
        case BUZZ_OK: return "ok";
        case BUZZ_EINVAL: return "invalid argument or configuration";
        case BUZZ_ECAPACITY: return "cache or workspace capacity exceeded";
        case BUZZ_ESTATE: return "call not valid in the current state (prefill first)";
        case BUZZ_EHIP: return "HIP runtime error";
        case BUZZ_EUNSUPPORTED: return "shape, dtype or parameter not covered by the kernels";
    }
    return "unknown status";
}

}  // extern "C"
