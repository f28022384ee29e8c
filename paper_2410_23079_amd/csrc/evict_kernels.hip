// BeeHive eviction kernels (Sec. 3.3; the eviction branch of Alg. 1, Alg. 2):
//   segment_topk : one wavefront per (segment, unit) ranks the segment's accumulated scores and
//                  emits the top min(keep, len) rows in index order (ties -> lowest index, NaN lowest);
//   gather_rows  : packs K, V, score and position of selected rows into their destination
//                  (survivors behind the old region, sink / window at prefill, export in cache order).
// Every segment yields min(keep, len) rows, so a survivor's destination is
// segment * keep + (rank among the segment's survivors): a wave-level prefix sum over the keep mask.
#include "buzz_internal.h"

namespace buzz {
namespace {

constexpr int kSelWaves = 4;

__global__ __launch_bounds__(256) void segment_topk_kernel(const SelectArgs a)
{
    extern __shared__ float lds[];                 // [kSelWaves][segment]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = blockIdx.x * kSelWaves + wave, unit = blockIdx.y;
    const int n_seg = (a.new_count + a.segment - 1) / a.segment;
    const bool active = seg < n_seg;
    const int start = seg * a.segment;
    const int len = active ? min(a.segment, a.new_count - start) : 0;
    const int take = min(a.keep, len);
    float* sc = lds + wave * a.segment;
    const float* base = a.score + (size_t)unit * a.unit_stride;
    for (int e = lane; e < len; e += 64) {
        const int row = a.lo + start + e;
        float v = a.ignore_scores ? 0.f : base[a.map.ring_cap ? a.map.phys(row) : row];   // all equal: lowest indices win
        if (v != v) v = -INFINITY;                 // NaN ranks below everything
        sc[e] = v;
    }
    __syncthreads();
    if (!active) return;
    int running = 0;
    for (int e0 = 0; e0 < len; e0 += 64) {
        const int e = e0 + lane;
        bool kp = false;
        if (e < len) {
            const float v = sc[e];
            int before = 0;                        // rows of the segment that rank strictly before row e
            for (int i = 0; i < len; ++i) {
                const float vi = sc[i];
                before += (vi > v) || (vi == v && i < e);
            }
            kp = before < take;
        }
        const unsigned long long mask = __ballot(kp);
        if (kp) {
            const int r = running + __popcll(mask & ((1ull << lane) - 1ull));
            a.sel[(size_t)unit * a.sel_stride + seg * a.keep + r] = a.lo + start + e;
        }
        running += __popcll(mask);
    }
}

// Segments too long for one wave's slice of the LDS (and the single segment of the H2O-style variant, which
// spans every row between sink and window): one block per (segment, unit) finds the `take` largest scores by a
// radix select on the order-preserving integer image of the scores -- four passes of a 256-bin histogram in
// LDS, most significant byte first, each narrowing the candidates to one bin -- which ends with the key of the
// last survivor and the number of rows with exactly that key that still fit.  A final pass in index order keeps
// every row with a larger key and the first of the equal ones (ties go to the lowest index), and numbers the
// survivors with a block-wide prefix sum so that they come out in index order.  Same result as the wave kernel.
constexpr int kTopkBlock = 1024;

__device__ inline unsigned score_key(float v)      // larger score <=> larger key; NaN ranks with -inf; -0 == +0
{
    if (v != v) v = -INFINITY;
    const unsigned b = __float_as_uint(v + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// exclusive prefix count of `flag` over the block in thread order, and the block total (both via LDS `tmp`,
// one slot per wave plus one); every thread of the block must call it
__device__ inline int block_prefix(bool flag, int* tmp, int& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const unsigned long long m = __ballot(flag);
    if (lane == 0) tmp[wave] = __popcll(m);
    __syncthreads();
    int before = 0, sum = 0;
    for (int w = 0; w < nw; ++w) { const int c = tmp[w]; before += w < wave ? c : 0; sum += c; }
    __syncthreads();                               // tmp is reused by the next call
    total = sum;
    return before + __popcll(m & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(kTopkBlock) void segment_topk_block_kernel(const SelectArgs a)
{
    __shared__ int hist[256];
    __shared__ int tmp[kTopkBlock / 64];
    __shared__ unsigned sh_prefix;
    __shared__ int sh_remaining;
    const int tid = threadIdx.x, seg = blockIdx.x, unit = blockIdx.y;
    const long long start = (long long)seg * a.segment;
    const int len = (int)min((long long)a.segment, (long long)a.new_count - start);
    const int take = min(a.keep, len);
    if (take <= 0) return;
    const float* base = a.score + (size_t)unit * a.unit_stride;
    auto key_of = [&](int e) {
        const int row = a.lo + (int)start + e;
        return a.ignore_scores ? 0x80000000u : score_key(base[a.map.ring_cap ? a.map.phys(row) : row]);
    };
    // radix select: after the pass for byte b, `prefix` holds the top bytes of the last survivor's key and
    // `remaining` how many rows are still to be taken among those that share them
    unsigned prefix = 0, mask = 0;
    int remaining = take;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int e = tid; e < len; e += kTopkBlock) {
            const unsigned k = key_of(e);
            if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid == 0) {
            int left = remaining, bin = 255;
            for (; bin > 0; --bin) {               // from the largest digit down: the bin where the count runs out
                if (hist[bin] >= left) break;
                left -= hist[bin];
            }
            sh_prefix = prefix | ((unsigned)bin << shift);
            sh_remaining = left;
        }
        __syncthreads();
        prefix = sh_prefix; remaining = sh_remaining;
        mask |= 255u << shift;
        __syncthreads();
    }
    // prefix = key of the last survivor; `remaining` (>= 1) rows with that key survive, the lowest indices first
    int ties_seen = 0, kept_seen = 0;
    int* out = a.sel + (size_t)unit * a.sel_stride + (size_t)seg * a.keep;
    for (int e0 = 0; e0 < len; e0 += kTopkBlock) {
        const int e = e0 + tid;
        const unsigned k = e < len ? key_of(e) : 0u;
        const bool eq = e < len && k == prefix, gt = e < len && k > prefix;
        int n_eq, n_kp;
        const int eq_before = ties_seen + block_prefix(eq, tmp, n_eq);
        const bool kp = gt || (eq && eq_before < remaining);
        const int pos = kept_seen + block_prefix(kp, tmp, n_kp);
        if (kp) out[pos] = a.lo + (int)start + e;
        ties_seen += n_eq; kept_seen += n_kp;
    }
}

// Eviction of the new rows in one launch, for caches whose old rows stay in place.  A wave ranks one segment
// as above and then moves the segment's survivors itself (their destination depends on nothing but the
// segment number and the rank).  A score update that the last decode step left pending is applied on the fly
// to the rows of the segment -- nothing else needs it now: every other retained row keeps its physical place,
// and the next decode step applies the update there as it would have without an eviction.  A survivor arrives
// with its updated score, and its entry in that step's logit buffer is set to -inf so that the next step
// adds exactly 0 for it.
__global__ __launch_bounds__(256) void evict_new_rows_kernel(const EvictArgs a)
{
    extern __shared__ float lds[];                 // [kSelWaves][segment] scores, then [kSelWaves][keep] kept offsets
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = blockIdx.x * kSelWaves + wave, unit = blockIdx.y;
    const int n_seg = (a.new_count + a.segment - 1) / a.segment;
    if (seg >= n_seg) return;                      // no block-wide barrier below: a wave only reads what it wrote
    const int start = seg * a.segment;
    const int len = min(a.segment, a.new_count - start);
    const int take = min(a.keep, len);
    float* sc = lds + wave * a.segment;
    int* kept = (int*)(lds + kSelWaves * a.segment) + wave * a.keep;
    const size_t ubase = (size_t)unit * a.cap;
    const float* logit_u = a.logit_prev ? a.logit_prev + ubase * a.G : nullptr;
    auto current_score = [&](int ph) {             // the row's score with the pending update applied
        float v = a.score[ubase + ph];
        if (logit_u)
            for (int g = 0; g < a.G; ++g)
                v = add_probability(v, logit_u[(size_t)g * a.cap + ph], a.stat_prev[((size_t)unit * a.G + g) * 2],
                                    a.stat_prev[((size_t)unit * a.G + g) * 2 + 1]);
        return v;
    };
    for (int e = lane; e < len; e += 64) {
        float v = a.ignore_scores ? 0.f : current_score(a.map.phys(a.lo + start + e));   // all equal: lowest indices win
        if (v != v) v = -INFINITY;                 // NaN ranks below everything
        sc[e] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    int running = 0;
    for (int e0 = 0; e0 < len; e0 += 64) {
        const int e = e0 + lane;
        bool kp = false;
        if (e < len) {
            const float v = sc[e];
            int before = 0;                        // rows of the segment that rank strictly before row e
            for (int i = 0; i < len; ++i) {
                const float vi = sc[i];
                before += (vi > v) || (vi == v && i < e);
            }
            kp = before < take;
        }
        const unsigned long long mask = __ballot(kp);
        if (kp) kept[running + __popcll(mask & ((1ull << lane) - 1ull))] = e;
        running += __popcll(mask);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // move the survivors: 16 bytes per lane, 64 / lpr rows per pass
    const int lpr = a.row_bytes >> 4;              // lanes per row (at most 64)
    const int c = lane % lpr, rr = lane / lpr, rows_per_pass = 64 / lpr;
    for (int r = rr; r < take; r += rows_per_pass) {
        const int sp = a.map.phys(a.lo + start + kept[r]);
        const int dp = a.dst_start + seg * a.keep + r;
        const size_t so = (ubase + sp) * a.row_bytes + c * 16, dof = (ubase + dp) * a.row_bytes + c * 16;
        *(uint4*)((char*)a.K + dof) = *(const uint4*)((const char*)a.K + so);
        *(uint4*)((char*)a.V + dof) = *(const uint4*)((const char*)a.V + so);
        if (c == 0) {
            a.score[ubase + dp] = current_score(sp);
            a.pos[ubase + dp] = a.pos[ubase + sp];
            if (a.logit_prev)
                for (int g = 0; g < a.G; ++g) a.logit_prev[ubase * a.G + (size_t)g * a.cap + dp] = -INFINITY;
        }
    }
}

constexpr int kGatherRowsPerBlock = 64;

__global__ __launch_bounds__(256) void gather_rows_kernel(const GatherArgs a)
{
    const int unit = blockIdx.y, tid = threadIdx.x;
    const int lpr = a.row_bytes >> 4;              // 16-byte lanes per row
    const int c = tid % lpr, rr = tid / lpr, rows_per_pass = 256 / lpr;
    const int rbeg = blockIdx.x * kGatherRowsPerBlock;
    const int rend = min(a.n_rows, rbeg + kGatherRowsPerBlock);
    const size_t sbase = (size_t)unit * a.src_unit_rows, dbase = (size_t)unit * a.dst_unit_rows;
    for (int r = rbeg + rr; r < rend; r += rows_per_pass) {
        const int src = a.sel ? a.sel[(size_t)unit * a.sel_stride + a.sel_start + (size_t)r * a.sel_step]
                              : a.src_start + r * a.src_step;
        const int sp = a.src_map.ring_cap ? a.src_map.phys(src) : src;
        const size_t so = (sbase + sp) * a.row_bytes + c * 16;
        const size_t dro = dbase + a.dst_start + r;
        const size_t dof = dro * a.row_bytes + c * 16;
        if (a.dstK) *(uint4*)((char*)a.dstK + dof) = *(const uint4*)((const char*)a.srcK + so);
        if (a.dstV) *(uint4*)((char*)a.dstV + dof) = *(const uint4*)((const char*)a.srcV + so);
        if (c == 0) {
            if (a.dstScore) a.dstScore[dro] = a.srcScore[sbase + sp];
            if (a.dstPos) a.dstPos[dro] = a.srcPos ? a.srcPos[sbase + sp] : src;
        }
    }
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float* dst, const float* src, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src ? src[i] : 0.f;
}

__global__ __launch_bounds__(256) void plain_copy_kernel(uint4* dst, const uint4* src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_plain_copy(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(plain_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint4*)dst, (const uint4*)src, n16);
    return hipGetLastError();
}

hipError_t launch_evict_new_rows(const EvictArgs& a, int units, hipStream_t st, Timing tm)
{
    const int n_seg = (a.new_count + a.segment - 1) / a.segment;
    if (n_seg <= 0 || a.keep <= 0) return hipSuccess;
    if (a.row_bytes > 1024 || (a.row_bytes & 15) || 64 % (a.row_bytes >> 4)) return hipErrorInvalidValue;
    const dim3 grid((n_seg + kSelWaves - 1) / kSelWaves, units);
    const size_t lds = (size_t)kSelWaves * (a.segment + a.keep) * sizeof(float);
    BUZZ_LAUNCH(evict_new_rows_kernel, grid, dim3(256), lds, st, tm, a);
    return hipGetLastError();
}

hipError_t launch_segment_topk(const SelectArgs& a, int units, hipStream_t st, Timing tm)
{
    const int n_seg = (a.new_count + a.segment - 1) / a.segment;
    if (n_seg <= 0) return hipSuccess;
    if (a.segment > kMaxWaveSegment) {             // a segment's scores no longer fit a wave's slice of the LDS
        if (n_seg > 65535) return hipErrorInvalidValue;
        BUZZ_LAUNCH(segment_topk_block_kernel, dim3(n_seg, units), dim3(kTopkBlock), 0, st, tm, a);
        return hipGetLastError();
    }
    dim3 grid((n_seg + kSelWaves - 1) / kSelWaves, units), block(256);
    const size_t lds = (size_t)kSelWaves * a.segment * sizeof(float);
    BUZZ_LAUNCH(segment_topk_kernel, grid, block, lds, st, tm, a);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const GatherArgs& a, int units, hipStream_t st, Timing tm)
{
    if (a.n_rows <= 0) return hipSuccess;
    dim3 grid((a.n_rows + kGatherRowsPerBlock - 1) / kGatherRowsPerBlock, units), block(256);
    BUZZ_LAUNCH(gather_rows_kernel, grid, block, 0, st, tm, a);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float* dst, const float* src, int64_t n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, dst, src, n);
    return hipGetLastError();
}

}  // namespace buzz
