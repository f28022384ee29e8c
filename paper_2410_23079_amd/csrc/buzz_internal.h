// Internal declarations shared by the host API and the HIP kernels of the BUZZ decode library.
//
// Physical layout of one (batch, kv-head) unit, `cap` rows:
//
//     [ sink k | old region (old_cap rows, grows upward) | ring of R = w + T rows ]
//       0        k                                          ring_base = cap - R
//
// Attention is invariant under a permutation of the cache rows (eq. 3 is a sum over rows), so
// the "new + window" tail of the paper's cache order lives in a ring: a decode step appends at
// the ring's tail, an eviction copies the survivors of the oldest tail rows to the end of the
// old region and advances the ring head.  The window never moves.  Logical (paper) order is
//     row j <  front : physical row j                      (front = sink rows filled + n_old)
//     row j >= front : physical row ring_base + (head + j - front) mod R
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "buzz.h"

namespace buzz {

constexpr int kMaxSplits = 128;        // upper bound on key-range splits per unit
constexpr int kDefaultCUs = 256;       // MI355X; replaced by the device's own count at the first launch
constexpr int kMaxBlocks = 4096;       // partial buffers are sized for units * splits <= this (or 1 split per unit)
constexpr int kMaxWaveSegment = 4096;  // longest segment the one-wave-per-segment selection kernels rank (LDS slice)
constexpr int kMinSplitRows = 128;     // automatic split policy: no split shorter than this
constexpr int kStageFloats = 4096;     // LDS logit staging of one split that every shape can have
constexpr int kStageFloatsMax = 8192;  // ... and what a shape gets when the block's other LDS arrays leave room

// 8-wave decode blocks only below this group size * head_dim: eight waves' partial outputs (32 bytes per
// element) and kStageFloats of logit staging must fit 64 KB of LDS
constexpr int kWideBlockMaxGD = 1505;

// Floats of LDS staging (rows_per_split * group size) a decode block may use: as much as keeps the block's
// LDS (the waves' partial outputs [waves][G][D] and running statistics, the staging) within 64 KB, between
// kStageFloats and kStageFloatsMax.  A larger staging area lets one split cover a longer row range, so a
// unit needs fewer splits; the workspace bound on the split count assumes kStageFloats.
inline int stage_floats(int G, int D)
{
    const int waves = G * D < kWideBlockMaxGD ? 8 : 4;
    const int fixed = waves * G * D * 4 + 2 * 8 * G * 4 + 64;
    int f = (65536 - fixed) / 4;
    if (f > kStageFloatsMax) f = kStageFloatsMax;
    if (f < kStageFloats) f = kStageFloats;
    return f;
}
constexpr double kLastLevelCacheBytes = 256.0 * 1024 * 1024;   // Infinity Cache of one MI355X      // segment scores of one wave must fit its LDS slice

struct RingMap {
    int32_t front;      // rows [0, front) are stored linearly
    int32_t ring_base;  // first physical row of the ring
    int32_t ring_head;  // ring offset of logical row `front`
    int32_t ring_cap;   // R
    __host__ __device__ inline int32_t phys(int32_t j) const {
        if (j < front) return j;
        int32_t r = ring_head + (j - front);
        if (r >= ring_cap) r -= ring_cap;
        return ring_base + r;
    }
};

struct AttnArgs {
    const void* q;       // [B][Hq][D]
    const void* k_new;   // [B][Hkv][D]
    const void* v_new;
    void* K;             // [units][cap][D]
    void* V;
    float* score;        // [units][cap]
    int32_t* pos;        // [units][cap]
    float* logit;        // [units][G][cap]  scaled logits in log2 units, written by this step
    const float* logit_prev;  // same layout: the previous step's logits (valid when pending)
    float* part_ml;      // [units][s_cap][G][2]  (running max, running sum) per split
    float* part_o;       // [units][s_cap][G][D]  unnormalised partial outputs per split
    float* stat;         // [units][G][2]  this step's global (max, 1/sum), written by the merging block
    const float* stat_prev;   // the previous step's
    int32_t* ticket;     // [units] arrival counters, zero between launches
    float* out;          // [B][Hq][D]
    RingMap map;
    int32_t n;           // retained rows including the one being appended (logical index n-1)
    int32_t new_phys;    // physical row the appended token is written to
    int32_t new_pos;     // its original token index
    int32_t cap;
    int32_t rows_per_split;
    int32_t n_splits;
    int32_t s_cap;
    int32_t Hq, Hkv;
    int32_t waves;       // waves per block: 4, or 8 when every unit is a single split
    int32_t pending;     // 1: the previous step's score update has not been applied yet
    int32_t streaming;   // 1: K/V are read with the non-temporal hint (working set exceeds the last-level cache)
    int32_t fixed_tiles; // 1: waves take tiles in a fixed round-robin (bitwise reproducible results)
    int32_t xcd_local;   // 1: blocks are renumbered so that a unit's splits share one die, and merge through its L2
    uint32_t die_map;    // ... and the die (4 bits each) that serves launch-order block numbers 0..7 mod 8
    float scale_log2;    // softmax scale * log2(e)
};

// The lazy score update of one row and head: score + exp2(logit - max) / sum of the step that left it pending.
// One definition for every kernel that applies it (the next decode step, the flush, the eviction), so that
// whichever of them does, the bits are the same.
__device__ inline float add_probability(float score, float logit, float row_max, float inv_sum)
{
    return fmaf(__builtin_amdgcn_exp2f(logit - row_max), inv_sum, score);
}

struct SelectArgs {
    const float* score;        // base of the score array the segments live in
    int64_t unit_stride;       // elements between units in `score`
    RingMap map;               // mapping of logical rows (ring_cap == 0: identity)
    int32_t lo;                // logical index of the first new row
    int32_t new_count;         // rows to segment
    int32_t segment, keep;
    int32_t ignore_scores;     // ablation: keep the first `keep` rows of every segment (interval sampling)
    int32_t* sel;              // [units][sel_stride] logical source rows of the survivors, increasing
    int32_t sel_stride;
};

// Eviction of the new rows when the old rows stay where they are (old stride 1): segmented top-c and the
// survivors' move in one launch.
struct EvictArgs {
    void* K; void* V;          // [units][cap][row_bytes]
    float* score;              // [units][cap]
    int32_t* pos;              // [units][cap]
    float* logit_prev;         // [units][G][cap] logits of the last decode step, NULL when no score update is pending
    const float* stat_prev;    // [units][G][2] its (max, 1 / sum)
    RingMap map;               // logical -> physical rows before the eviction
    int32_t lo;                // logical index of the first new row
    int32_t new_count;         // rows to segment
    int32_t segment, keep;
    int32_t ignore_scores;     // ablation: keep the first `keep` rows of every segment
    int32_t dst_start;         // physical (= logical) row the first survivor moves to
    int32_t cap, row_bytes, G;
};

struct GatherArgs {
    const void* srcK; const void* srcV; const float* srcScore; const int32_t* srcPos;  // srcPos NULL => pos = source row
    int64_t src_unit_rows;     // rows between units in the source arrays
    RingMap src_map;           // ring_cap == 0: identity
    const int32_t* sel;        // NULL => affine source rows
    int32_t sel_stride, sel_start, sel_step;
    int32_t src_start, src_step;
    void* dstK; void* dstV; float* dstScore; int32_t* dstPos;    // any may be NULL
    int64_t dst_unit_rows;
    int32_t dst_start;
    int32_t n_rows;
    int32_t row_bytes;         // D * sizeof(element)
};

struct ObsArgs {               // prefill scoring: causal attention of observed prompt queries (one pass)
    const void* K;             // [units][N][D]
    const void* q_obs;         // [B][Hq][n_obs][D]; query t sits at prompt position N - n_obs + t
    float* score;              // [units][N]   accumulated in place
    float* stats;              // vector path: [units][key_blocks][kObsRows][2] per key-block (max, sum) of every query
                               // row; matrix-core path: [B * Hq][key_splits][kObsPassRows][2] (reference, sum) of
                               // every query over each part of its keys
    int32_t N, n_obs;
    int32_t t_begin, t_count;  // queries scored by this pass; at most obs_pass_queries()
    int32_t Hq, Hkv;
    int32_t log_n;             // 1: a query at prompt position i is scaled by log(i + 1) / log(512) (Sec. 3.5)
    int32_t key_splits;        // matrix-core path: blocks that share the keys of one group of 256 queries (1..kObsKeySplits)
    float scale_log2;
};

constexpr int kObsRows = 256;        // query rows (query x group member) per pass = threads per block
constexpr int kObsKeyBlock = 1024;   // keys per block of the row-statistics kernel
constexpr int kObsPassRows = 4096;   // matrix-core scoring: queries per head and pass
constexpr int kObsKeySplits = 4;     // ... and the most blocks that share one query group's keys

// Optional event pair: when both are non-null the launch records the kernel's own begin / end
// timestamps into them (used by the benchmark profiling pass).
struct Timing { hipEvent_t begin = nullptr, end = nullptr; };

#define BUZZ_LAUNCH(kernel, grid, block, lds, st, tm, ...)                                            \
    do {                                                                                               \
        if ((tm).begin) hipExtLaunchKernelGGL(kernel, grid, block, lds, st, (tm).begin, (tm).end, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                            \
    } while (0)

hipError_t launch_attn_split(int dtype, int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm = {});
hipError_t launch_flush_scores(int G, const AttnArgs& a, int units, hipStream_t st, Timing tm = {});
hipError_t launch_segment_topk(const SelectArgs& a, int units, hipStream_t st, Timing tm = {});
hipError_t launch_gather_rows(const GatherArgs& a, int units, hipStream_t st, Timing tm = {});
hipError_t launch_fill_f32(float* dst, const float* src, int64_t n, hipStream_t st);  // src NULL => zeros
hipError_t launch_plain_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
hipError_t launch_evict_new_rows(const EvictArgs& a, int units, hipStream_t st, Timing tm = {});
hipError_t launch_obs_scores(int dtype, int D, int G, const ObsArgs& a, int units, hipStream_t st, Timing tm = {});
int obs_pass_queries(int dtype, int G);   // queries of one head a single scoring pass covers
int attn_tile_rows(int dtype, int D, int G);   // rows one block consumes per loop trip (split sizes are multiples)
bool attn_supported(int dtype, int D, int G);

}  // namespace buzz
