// Decode attention over the retained BUZZ cache (eq. 3 / eq. 5 of the paper) as ONE kernel per step:
// the append of eq. 2, the split-softmax attention, the merge of the splits and the accumulated-score
// update ("A" of Alg. 2) all happen inside attn_split.
//
//  - One block per (key-range split, unit).  A wave reads 64 x 16 B per load instruction = RPW
//    consecutive cache rows, LPR = 64 / RPW lanes per row: every load is one contiguous 1 KB burst.
//    q.k is a two-element-dot chain per lane plus an LPR-lane DPP reduction; softmax runs online per
//    lane group; p.V accumulates in registers.
//  - The scaled logit of every row is written to a scratch array.  A row's probability needs the
//    maximum and sum over ALL splits, which only exist once the step is over, so the score update of
//    step t is applied by step t+1 while it streams the same rows anyway (one lane per row, coalesced):
//    score += sum_g exp2(logit_t - M_t[g]) / L_t[g].  flush_scores applies a pending update right away;
//    the host calls it before anything reads the scores (eviction, export).
//  - The block that finishes last for a unit (atomic ticket, nobody waits) merges the split partials
//    into the attention output and publishes (M, 1/L) for the next step's score update.
#include <type_traits>

#include "buzz_internal.h"

namespace buzz {
namespace {

struct bf16_t { uint16_t x; };
struct fp16_t { uint16_t x; };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Build-time tuning knobs (defaults are the measured best; a sweep overrides them with -D).
#ifndef BUZZ_U_G1
#define BUZZ_U_G1 4      // 16-byte loads of K (and of V) per lane and tile, group size 1 (two tiles in flight)
#endif
#ifndef BUZZ_U_G2
#define BUZZ_U_G2 4
#endif
#ifndef BUZZ_U_G4
#define BUZZ_U_G4 4
#endif
#ifndef BUZZ_U_G8
#define BUZZ_U_G8 2
#endif
#ifndef BUZZ_MIN_BLOCKS
#define BUZZ_MIN_BLOCKS 1  // second argument of __launch_bounds__
#endif

template <typename T> struct Elem;
// cvt: 16 bytes -> VEC floats.  dot: sum over the 16 bytes of q * k in fp32 (16-bit types use the
// two-element dot instruction on the raw words: exact products, fp32 accumulation, no conversion).
template <> struct Elem<float> {
    static constexpr int VEC = 4;
    static __device__ inline void cvt(const u32x4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    static __device__ inline float dot(const u32x4& q, const u32x4& k) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) d = fmaf(__uint_as_float(q[i]), __uint_as_float(k[i]), d);
        return d;
    }
};
template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ inline void cvt(const u32x4& r, float* f) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(r[i] << 16);
            f[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
        }
    }
    static __device__ inline float dot(const u32x4& q, const u32x4& k) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, (unsigned int)q[i]),
                                                __builtin_bit_cast(bf16x2_t, (unsigned int)k[i]), d, false);
        return d;
    }
};
template <> struct Elem<fp16_t> {
    static constexpr int VEC = 8;
    static __device__ inline void cvt(const u32x4& r, float* f) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2_t h = __builtin_bit_cast(half2_t, (unsigned int)r[i]);
            f[2 * i] = (float)h.x;
            f[2 * i + 1] = (float)h.y;
        }
    }
    static __device__ inline float dot(const u32x4& q, const u32x4& k) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            d = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, (unsigned int)q[i]),
                                       __builtin_bit_cast(half2_t, (unsigned int)k[i]), d, false);
        return d;
    }
};

// NT: streaming hint for data that will not be re-read before it would be evicted anyway
template <bool NT> __device__ inline u32x4 load16(const char* p) {
    if constexpr (NT) return __builtin_nontemporal_load((const u32x4*)p);
    else return *(const u32x4*)p;
}

template <int CTRL> __device__ inline float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Sum over the LPR consecutive lanes that share a cache row; every lane of the group gets the total.
template <int LPR> __device__ inline float row_sum(float v) {
    v += dpp_move<0xB1>(v);                 // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);                 // quad_perm [2,3,0,1]
    if (LPR >= 8) v += dpp_move<0x141>(v);  // row_half_mirror
    if (LPR >= 16) v += dpp_move<0x140>(v); // row_mirror
    if (LPR >= 32) v += __shfl_xor(v, 16);
    if (LPR >= 64) v += __shfl_xor(v, 32);
    return v;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Split partials travel between blocks (possibly on different XCDs, each with its own L2) inside one
// launch.  They are written and read with device-scope atomic accesses, which go through to the
// memory side instead of staying in an XCD's L2, so no cache write-back or invalidate is needed.
__device__ inline void publish(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ inline float acquire(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Where a block works: logical rows [j0, j1) of one unit.  The range is cut into at most four physically
// contiguous runs (linear region, ring before the wrap, ring after the wrap, the row being appended).
struct SplitCtx {
    int split, unit, b, kvh;
    int j0, j1, jl1, wrap;
    size_t ubase;
};

__device__ inline SplitCtx make_ctx(const AttnArgs& a)
{
    SplitCtx x;
    x.split = blockIdx.x; x.unit = blockIdx.y;
    x.b = x.unit / a.Hkv; x.kvh = x.unit - x.b * a.Hkv;
    x.j0 = x.split * a.rows_per_split;
    x.j1 = min(a.n, x.j0 + a.rows_per_split);
    x.jl1 = min(x.j1, a.n - 1);                           // rows already stored in the arena end here
    x.wrap = a.map.front + a.map.ring_cap - a.map.ring_head;   // first logical row after the ring wraps
    x.ubase = (size_t)x.unit * a.cap;
    return x;
}

// run r covers logical rows [lo, hi) stored at physical rows phys0 ...; run 3 is the row being appended
__device__ inline void run_bounds(const AttnArgs& a, const SplitCtx& x, int run, int& lo, int& hi, int& phys0)
{
    if (run == 0) { lo = x.j0; hi = min(x.jl1, a.map.front); phys0 = lo; }
    else if (run == 1) { lo = max(x.j0, a.map.front); hi = min(x.jl1, x.wrap); phys0 = a.map.ring_base + a.map.ring_head + (lo - a.map.front); }
    else if (run == 2) { lo = max(x.j0, x.wrap); hi = x.jl1; phys0 = a.map.ring_base + (lo - x.wrap); }
    else { lo = a.n - 1; hi = x.j1 == a.n ? a.n : lo; phys0 = a.new_phys; }
}

// Everything a block does once its waves have put their (max, sum, unnormalised output) into LDS.
// The order hides as much latency as it can behind work that does not depend on it:
//   1. request what the side phase needs (previous logits, old scores) -- nothing is waiting for it yet;
//   2. merge the waves, publish the split's partial (write-through stores);
//   3. side phase: this step's logits leave LDS, the previous step's score update is applied;
//   4. wait for the published stores, synchronise, take the ticket;
//   5. the block that drew the last ticket merges all splits with ONE round of device-scope loads.
// sm_ml is scratch for step 5: [2][kMaxSplits][G] floats.
template <int G, int D, int NW>
__device__ inline void finish_split(const AttnArgs& a, const SplitCtx& x, const float* stage,
                                    float (*sm_m)[G], float (*sm_l)[G], float (*sm_acc)[G][D], float* sm_ml,
                                    int* sm_ticket)
{
    constexpr int NTHR = NW * 64;                         // threads per block
    const int tid = threadIdx.x;
    const int unit = x.unit, j0 = x.j0;
    const int S = a.n_splits;
    float* logit_u = a.logit + x.ubase * G;               // [G][cap] for this unit, written by this step
    const float* logit_prev_u = a.logit_prev + x.ubase * G;   // the previous step's logits
    float* score_u = a.score + x.ubase;
    float Mp[G], iLp[G];                                   // previous step's global max and 1/sum per head
#pragma unroll
    for (int g = 0; g < G; ++g) {
        Mp[g] = a.pending ? a.stat_prev[((size_t)unit * G + g) * 2] : 0.f;
        iLp[g] = a.pending ? a.stat_prev[((size_t)unit * G + g) * 2 + 1] : 0.f;
    }

    // 1. side-phase inputs of the first pass (4 rows per thread) of each stored run
    float4 pre_sc[3], pre_lp[3][G];
#pragma unroll
    for (int run = 0; run < 3; ++run) {
        int lo, hi, phys0;
        run_bounds(a, x, run, lo, hi, phys0);
        const int lead = phys0 & 3, pa = phys0 - lead, cnt = hi - lo + lead;
        if (a.pending && hi - lo > 0 && 4 * tid < cnt) {
            pre_sc[run] = *(const float4*)(score_u + pa + 4 * tid);
#pragma unroll
            for (int g = 0; g < G; ++g) pre_lp[run][g] = *(const float4*)(logit_prev_u + (size_t)g * a.cap + pa + 4 * tid);
        }
    }

    // 2. merge the waves; the only split writes the result, otherwise publish the partial
    __syncthreads();
    float* outp = a.out + (size_t)(x.b * a.Hq + x.kvh * G) * D;
    const size_t pbase = ((size_t)unit * a.s_cap + x.split) * G;
    for (int i = tid; i < G * D; i += NTHR) {
        const int g = i / D, d = i - g * D;
        float M = sm_m[0][g];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][g]);
        const float mref = (M == -INFINITY) ? 0.f : M;
        float o = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float wgt = fast_exp2(sm_m[w][g] - mref);
            o = fmaf(wgt, sm_acc[w][g][d], o);
            L = fmaf(wgt, sm_l[w][g], L);
        }
        if (S == 1) {
            outp[(size_t)g * D + d] = o / L;
            if (d == 0) {
                a.stat[((size_t)unit * G + g) * 2] = M;
                a.stat[((size_t)unit * G + g) * 2 + 1] = 1.0f / L;
            }
        } else {
            publish(a.part_o + (pbase + g) * D + d, o);
            if (d == 0) {
                publish(a.part_ml + (pbase + g) * 2, M);
                publish(a.part_ml + (pbase + g) * 2 + 1, L);
            }
        }
    }

    // 3. dense side phase, after the read stream of this block is over (the logits staged by all waves are
    // visible after the barrier above).  Four consecutive physical rows per thread, 16-byte accesses where
    // the whole group belongs to this split; the appended row starts from score 0.
    // (Doing the score update at the start of the block instead, under the latency of the first K/V
    // loads, was measured 8% slower: its writes then compete with the ramping read stream.)
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        int lo, hi, phys0;
        run_bounds(a, x, run, lo, hi, phys0);
        if (hi - lo <= 0) continue;
        const bool fresh = run == 3;
        const bool upd = a.pending && !fresh;
        const int lead = phys0 & 3, pa = phys0 - lead, cnt = hi - lo + lead;
        for (int r0 = 4 * tid; r0 < cnt; r0 += 4 * NTHR) {
            const int ph = pa + r0;
            float4 sc = make_float4(0.f, 0.f, 0.f, 0.f);
            if (upd) {
                float4 lp[G];
                if (run < 3 && r0 == 4 * tid) {           // first pass: requested in step 1
                    sc = pre_sc[run < 3 ? run : 0];
#pragma unroll
                    for (int g = 0; g < G; ++g) lp[g] = pre_lp[run < 3 ? run : 0][g];
                } else {
                    sc = *(const float4*)(score_u + ph);
#pragma unroll
                    for (int g = 0; g < G; ++g) lp[g] = *(const float4*)(logit_prev_u + (size_t)g * a.cap + ph);
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    sc.x += fast_exp2(lp[g].x - Mp[g]) * iLp[g];
                    sc.y += fast_exp2(lp[g].y - Mp[g]) * iLp[g];
                    sc.z += fast_exp2(lp[g].z - Mp[g]) * iLp[g];
                    sc.w += fast_exp2(lp[g].w - Mp[g]) * iLp[g];
                }
            }
            const int sj = lo - j0 + r0 - lead;           // staging index of the group's first row
            if (r0 >= lead && r0 + 3 < cnt) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float* sg = stage + g * a.rows_per_split + sj;
                    *(float4*)(logit_u + (size_t)g * a.cap + ph) = make_float4(sg[0], sg[1], sg[2], sg[3]);
                }
                if (upd || fresh) *(float4*)(score_u + ph) = sc;
            } else {                                      // ragged edge of the run: row by row
                const float scv[4] = {sc.x, sc.y, sc.z, sc.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (r0 + e >= lead && r0 + e < cnt) {
#pragma unroll
                        for (int g = 0; g < G; ++g) logit_u[(size_t)g * a.cap + ph + e] = stage[g * a.rows_per_split + sj + e];
                        if (upd || fresh) score_u[ph + e] = scv[e];
                    }
                }
            }
        }
    }
    if (S == 1) return;

    // 4. ticket: the block that arrives last for this unit sees every split's partial.  Every wave first
    // waits until its own published (write-through) stores have been acknowledged (vmcnt(0)), then the
    // block synchronises, then one thread takes the ticket: the ticket can never overtake a partial.
    // No cache maintenance is involved.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0), expcnt / lgkmcnt untouched
    __syncthreads();
    if (tid == 0) *sm_ticket = __hip_atomic_fetch_add(a.ticket + unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*sm_ticket != S - 1) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (tid == 0) __hip_atomic_store(a.ticket + unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next step

    // 5. merge the splits: every load of the first 16 splits is issued before anything waits
    constexpr int OPT = (G * D + NTHR - 1) / NTHR;              // output elements per thread
    constexpr int CH = 16;                                // splits per round of loads
    const float* ml = a.part_ml + (size_t)unit * a.s_cap * G * 2;
    const float* po = a.part_o + (size_t)unit * a.s_cap * G * D;
    float mlv[(2 * kMaxSplits * G + NTHR - 1) / NTHR];
#pragma unroll
    for (int k = 0; k < (int)(sizeof(mlv) / sizeof(float)); ++k) {
        const int i = tid + NTHR * k;                     // element i of [S][G][2]
        mlv[k] = i < S * G * 2 ? acquire(ml + i) : 0.f;
    }
    float x0[OPT][CH];
#pragma unroll
    for (int r = 0; r < OPT; ++r) {
        const int i = tid + NTHR * r;
#pragma unroll
        for (int e = 0; e < CH; ++e) x0[r][e] = (i < G * D && e < S) ? acquire(po + (size_t)e * G * D + i) : 0.f;
    }
#pragma unroll
    for (int k = 0; k < (int)(sizeof(mlv) / sizeof(float)); ++k) {
        const int i = tid + NTHR * k;
        if (i < S * G * 2) sm_ml[(i & 1) * kMaxSplits * G + (i >> 1)] = mlv[k];   // [0]: max, [1]: sum, each [S][G]
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < OPT; ++r) {
        const int i = tid + NTHR * r;
        if (i >= G * D) continue;
        const int g = i / D;
        float M = -INFINITY;
        for (int sp = 0; sp < S; ++sp) M = fmaxf(M, sm_ml[sp * G + g]);   // finite: the appended row is always present
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            if (e < S) {
                const float w = fast_exp2(sm_ml[e * G + g] - M);
                L = fmaf(sm_ml[kMaxSplits * G + e * G + g], w, L);
                o = fmaf(w, x0[r][e], o);
            }
        }
        for (int sp = CH; sp < S; ++sp) {                 // beyond the first round: one more load each
            const float w = fast_exp2(sm_ml[sp * G + g] - M);
            L = fmaf(sm_ml[kMaxSplits * G + sp * G + g], w, L);
            o = fmaf(w, acquire(po + (size_t)sp * G * D + i), o);
        }
        outp[i] = o / L;
        if (i - g * D == 0) {
            a.stat[((size_t)unit * G + g) * 2] = M;
            a.stat[((size_t)unit * G + g) * 2 + 1] = 1.0f / L;
        }
    }
}

// Vector-ALU streaming kernel (any dtype; the choice for one query head per kv head).
template <typename T, int D, int G, int U, bool NT, int NW>
__global__ __launch_bounds__(NW * 64, BUZZ_MIN_BLOCKS) void attn_split_kernel(const AttnArgs a)
{
    using E = Elem<T>;
    constexpr int VEC = E::VEC;
    constexpr int LPR = D / VEC;          // lanes per cache row
    constexpr int RPW = 64 / LPR;         // rows per wave-wide load
    constexpr int ROWB = D * (int)sizeof(T);
    constexpr int WROWS = RPW * U;        // rows one wave consumes per trip
    static_assert(LPR >= 8 && LPR <= 64, "row must span 8..64 lanes");
    static_assert((WROWS & (WROWS - 1)) == 0, "tiles anchor at multiples of WROWS");

    extern __shared__ float stage[];                      // [G][rows_per_split] logits of this split's rows
    __shared__ float sm_m[NW][G], sm_l[NW][G];
    __shared__ float sm_acc[NW][G][D];
    __shared__ float sm_ml[2 * kMaxSplits * G];
    __shared__ int sm_ticket;

    const SplitCtx x = make_ctx(a);
    const int unit = x.unit, b = x.b, kvh = x.kvh, j0 = x.j0, j1 = x.j1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane % LPR, rs = lane / LPR;

    u32x4 qr[G];                                          // this lane's 16 bytes of every query head, raw
    {
        const char* qb = (const char*)a.q + (size_t)(b * a.Hq + kvh * G) * ROWB + c * 16;
#pragma unroll
        for (int g = 0; g < G; ++g) qr[g] = *(const u32x4*)(qb + (size_t)g * ROWB);
    }

    const size_t ubase = x.ubase;
    char* Kb = (char*)a.K + ubase * ROWB;                 // wave-uniform bases; lanes add 32-bit offsets
    char* Vb = (char*)a.V + ubase * ROWB;
    const unsigned lane_off = c * 16;

    float m[G], l[G], acc[G][VEC];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[g][v] = 0.f;
    }

    // Work split inside a block.  A split's logical row range is cut into at most four physically
    // contiguous runs; inside a run the block's waves take tiles of WROWS rows round-robin, on a grid
    // anchored at a physical multiple of WROWS (`lead` rows before the run's first row are masked).  The streaming phase only reads: logits are staged in LDS, and all per-row side
    // traffic (this step's logits out, the previous step's logits and the old score in, the new score out)
    // happens in one dense phase at the end of the block.  Writes that trickle into a saturated read
    // stream were measured to cost ~5% of the kernel per 1% of extra bytes.
    auto load_tile = [&](u32x4 (&kr)[U], u32x4 (&vr)[U], const char* kp, const char* vp, int base, int lead, int cnt) {
#pragma unroll
        for (int u = 0; u < U; ++u) {      // masked lanes re-read a valid row of the run
            const unsigned off = (unsigned)(min(max(base + u * RPW + rs, lead), cnt - 1) - lead) * ROWB + lane_off;
            kr[u] = load16<NT>(kp + off);
            vr[u] = load16<NT>(vp + off);
        }
    };

    // `stg` = staging index (row relative to the split's first row) of the tile's first row
    auto compute_tile = [&](const u32x4 (&kr)[U], const u32x4 (&vr)[U], int base, int lead, int cnt, int stg) {
        float s[G][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = base + u * RPW + rs;
            const bool ok = r >= lead && r < cnt;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float d = row_sum<LPR>(E::dot(qr[g], kr[u])) * a.scale_log2;
                s[g][u] = ok ? d : -INFINITY;
                if (c == 0 && ok) stage[g * a.rows_per_split + stg + u * RPW + rs] = d;
            }
        }
        // online softmax: s becomes the unnormalised probability relative to the running maximum
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float tmax = s[g][0];
#pragma unroll
            for (int u = 1; u < U; ++u) tmax = fmaxf(tmax, s[g][u]);
            const float mn = fmaxf(m[g], tmax);
            const float mref = (mn == -INFINITY) ? 0.f : mn;
            const float alpha = fast_exp2(m[g] - mref);
            m[g] = mn;
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                s[g][u] = fast_exp2(s[g][u] - mref);
                psum += s[g][u];
            }
            l[g] = fmaf(l[g], alpha, psum);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[g][v] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[VEC];
            E::cvt(vr[u], vf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[g][v] = fmaf(s[g][u], vf[v], acc[g][v]);
            }
        }
    };

    for (int run = 0; run < 4; ++run) {
        int lo, hi, phys0;
        run_bounds(a, x, run, lo, hi, phys0);
        if (hi - lo <= 0) continue;
        const char *kp, *vp;
        const int lead = phys0 & (WROWS - 1);             // rows between the aligned anchor and the run's first row
        const int cnt = hi - lo + lead;                   // run length measured from the anchor
        if (run < 3) {
            kp = Kb + (size_t)phys0 * ROWB;
            vp = Vb + (size_t)phys0 * ROWB;
        } else {                                          // eq. 2: the new row comes from the caller and joins the cache
            kp = (const char*)a.k_new + (size_t)unit * ROWB;
            vp = (const char*)a.v_new + (size_t)unit * ROWB;
            if (wave == 0 && rs == 0) {
                *(u32x4*)(Kb + (size_t)a.new_phys * ROWB + lane_off) = *(const u32x4*)(kp + lane_off);
                *(u32x4*)(Vb + (size_t)a.new_phys * ROWB + lane_off) = *(const u32x4*)(vp + lane_off);
                if (c == 0) a.pos[ubase + a.new_phys] = a.new_pos;
            }
        }
        // the block's waves take the run's tiles round-robin (a block-contiguous stream; measured ~5% faster
        // than giving every wave its own contiguous piece)
        constexpr int STEP = NW * WROWS;
        if constexpr (G == 1) {
        // two tile buffers: the next tile's loads are issued before the current tile is consumed
        u32x4 ka[U], va[U], kb[U], vb[U];
        int base = wave * WROWS;
        if (base < cnt) load_tile(ka, va, kp, vp, base, lead, cnt);
        while (base < cnt) {
            if (base + STEP < cnt) load_tile(kb, vb, kp, vp, base + STEP, lead, cnt);
            compute_tile(ka, va, base, lead, cnt, lo - j0 + base - lead);
            base += STEP;
            if (base >= cnt) break;
            if (base + STEP < cnt) load_tile(ka, va, kp, vp, base + STEP, lead, cnt);
            compute_tile(kb, vb, base, lead, cnt, lo - j0 + base - lead);
            base += STEP;
        }
        } else {
        for (int base = wave * WROWS; base < cnt; base += STEP) {
            u32x4 kr[U], vr[U];
            load_tile(kr, vr, kp, vp, base, lead, cnt);
            compute_tile(kr, vr, base, lead, cnt, lo - j0 + base - lead);
        }
        }
    }

    // merge the RPW lane groups of this wave (same columns, different rows)
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(m[g], off);
            const float lo = __shfl_xor(l[g], off);
            const float mn = fmaxf(m[g], mo);
            const float mref = (mn == -INFINITY) ? 0.f : mn;
            const float wa = fast_exp2(m[g] - mref), wb = fast_exp2(mo - mref);
            l[g] = l[g] * wa + lo * wb;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const float ao = __shfl_xor(acc[g][v], off);
                acc[g][v] = acc[g][v] * wa + ao * wb;
            }
            m[g] = mn;
        }
    }

    // merge the waves of the block through LDS and emit this split's partial
    if (rs == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) sm_acc[wave][g][c * VEC + v] = acc[g][v];
        }
        if (c == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
        }
    }
    (void)j1;
    finish_split<G, D, NW>(a, x, stage, sm_m, sm_l, sm_acc, sm_ml, &sm_ticket);
}

// ---------------------------------------------------------------------------------------------------
// Matrix-core streaming kernel for grouped queries (G >= 2 query heads per kv head, 16-bit cache).
// With several heads per cache row, q.K^T and p.V are small dense contractions; on the vector ALU they
// cost ~100 instructions per row pair and the kernel stops being bandwidth-bound.  Here a wave works
// on tiles of 16 cache rows with 16x16 MFMA tiles whose 16 "head" slots hold the G real heads:
//
//   S[row][head]  = K[16 rows x D] . Q^T[D x 16]       v_mfma_f32_16x16x32, D/32 instructions
//   O[head][d]   += P[16 x 16 rows] . V[16 rows x d]   v_mfma_f32_16x16x16, 8 column groups x (hi + lo)
//
// Lane l = (j = l % 16, q = l / 16).
//  * K operand: lane (j, q) holds row j of the tile, 16-byte chunks 4p + q, p = 0 .. D/32-1 (one load
//    instruction fetches 64 contiguous bytes of each of 16 rows).  The contraction index may be permuted
//    freely as long as Q uses the same permutation: lane (j, q) of the Q operand holds head j, the same
//    chunks (zero for j >= G).
//  * S comes out with lane (j, q) holding head j, rows 4q .. 4q+3: exactly the layout the P operand of
//    the second contraction needs, so softmax results go straight back into the matrix core.
//    P is split into a 16-bit head and a 16-bit remainder (two MFMAs) to keep ~16 bits of it.
//  * V operand: lane (j, q) needs rows 4q .. 4q+3 of one column.  It loads the 16-byte chunk j of those
//    four rows (each load instruction: four whole, contiguous rows) and transposes the 4 x 8 block in
//    registers, which yields the operands of 8 column groups; column group m of lane j is column 8j + m.
//  * O comes out with lane (j, q) holding heads 4q .. 4q+3 of its 8 columns.
template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    static __device__ inline f32x4 qk(const u32x4& k, const u32x4& q, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, k), __builtin_bit_cast(bf16x8_t, q), c, 0, 0, 0);
    }
    static __device__ inline f32x4 pv(const u32x2& p, const u32x2& v, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, p), __builtin_bit_cast(s16x4_t, v), c, 0, 0, 0);
    }
    static __device__ inline void split(float p, unsigned& hi, unsigned& lo) {   // p ~= hi + lo, both bf16
        const __bf16 h = (__bf16)p;
        hi = __builtin_bit_cast(unsigned short, h);
        lo = __builtin_bit_cast(unsigned short, (__bf16)(p - (float)h));
    }
};
template <> struct Mma<fp16_t> {
    static __device__ inline f32x4 qk(const u32x4& k, const u32x4& q, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, k), __builtin_bit_cast(f16x8_t, q), c, 0, 0, 0);
    }
    static __device__ inline f32x4 pv(const u32x2& p, const u32x2& v, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, p), __builtin_bit_cast(f16x4_t, v), c, 0, 0, 0);
    }
    static __device__ inline void split(float p, unsigned& hi, unsigned& lo) {
        const _Float16 h = (_Float16)p;
        hi = __builtin_bit_cast(unsigned short, h);
        lo = __builtin_bit_cast(unsigned short, (_Float16)(p - (float)h));
    }
};

template <typename T, int D, int G, bool NT, int NW>
__global__ __launch_bounds__(NW * 64) void attn_split_mfma_kernel(const AttnArgs a)
{
    constexpr int ROWB = D * 2;
    constexpr int NCH = D / 8;                            // 16-byte chunks per row
    constexpr int QP = NCH / 4;                           // K / Q chunks per lane
    constexpr int VS = (NCH + 15) / 16;                   // sets of 16 column chunks
    constexpr int WROWS = 16;
    static_assert(G >= 2 && G <= 16 && NCH % 4 == 0, "grouped queries, head_dim multiple of 32");

    extern __shared__ float stage[];                      // [G][rows_per_split] logits of this split's rows
    __shared__ float sm_m[NW][G], sm_l[NW][G];
    __shared__ float sm_acc[NW][G][D];
    __shared__ float sm_ml[2 * kMaxSplits * G];
    __shared__ int sm_ticket;

    const SplitCtx x = make_ctx(a);
    const int unit = x.unit, j0 = x.j0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;

    u32x4 qb[QP];                                         // Q operand: head j, chunks 4p + q
#pragma unroll
    for (int p = 0; p < QP; ++p) {
        qb[p] = u32x4{0u, 0u, 0u, 0u};
        if (j < G) qb[p] = *(const u32x4*)((const char*)a.q + (size_t)(x.b * a.Hq + x.kvh * G + j) * ROWB + (4 * p + q) * 16);
    }

    char* Kb = (char*)a.K + x.ubase * ROWB;
    char* Vb = (char*)a.V + x.ubase * ROWB;

    float m_run = -INFINITY, l_run = 0.f;                 // head j (replicated over q; l_run is this lane's share)
    f32x4 O[VS][8];                                       // heads 4q .. 4q+3 of columns 8 (16 t + j) + m
#pragma unroll
    for (int t = 0; t < VS; ++t) {
#pragma unroll
        for (int mcol = 0; mcol < 8; ++mcol) O[t][mcol] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    auto load_tile = [&](u32x4 (&kk)[QP], u32x4 (&vv)[VS][4], const char* kp, const char* vp, int base, int lead, int cnt) {
        const unsigned krow = (unsigned)(min(max(base + j, lead), cnt - 1) - lead) * ROWB;
#pragma unroll
        for (int p = 0; p < QP; ++p) kk[p] = load16<NT>(kp + krow + (4 * p + q) * 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned vrow = (unsigned)(min(max(base + 4 * q + e, lead), cnt - 1) - lead) * ROWB;
#pragma unroll
            for (int t = 0; t < VS; ++t) vv[t][e] = load16<NT>(vp + vrow + ((16 * t + j) % NCH) * 16);
        }
    };

    auto compute_tile = [&](const u32x4 (&kk)[QP], const u32x4 (&vv)[VS][4], int base, int lead, int cnt, int stg) {
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < QP; ++p) sacc = Mma<T>::qk(kk[p], qb[p], sacc);
        float s[4];
        float tmax = -INFINITY;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = base + 4 * q + v;
            const bool ok = r >= lead && r < cnt;
            const float d = sacc[v] * a.scale_log2;
            s[v] = ok ? d : -INFINITY;
            if (ok && j < G) stage[j * a.rows_per_split + stg + 4 * q + v] = d;
            tmax = fmaxf(tmax, s[v]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float mn = fmaxf(m_run, tmax);
        const float mref = (mn == -INFINITY) ? 0.f : mn;
        const float alpha = fast_exp2(m_run - mref);
        m_run = mn;
        unsigned hi[4], lo[4];
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float pr = fast_exp2(s[v] - mref);
            Mma<T>::split(pr, hi[v], lo[v]);
            psum += pr;
        }
        l_run = fmaf(l_run, alpha, psum);
        const u32x2 p_hi = {hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
        const u32x2 p_lo = {lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
        if (__any(alpha != 1.0f)) {                       // a running maximum moved: rescale the outputs
            float av[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) av[v] = __shfl(alpha, (4 * q + v) & 15);   // head 4q+v lives in lane 4q+v
#pragma unroll
            for (int t = 0; t < VS; ++t) {
#pragma unroll
                for (int mcol = 0; mcol < 8; ++mcol) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) O[t][mcol][v] *= av[v];
                }
            }
        }
#pragma unroll
        for (int t = 0; t < VS; ++t) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {                 // dword w of the chunk = columns 2w and 2w+1
                const unsigned r0 = vv[t][0][w], r1 = vv[t][1][w], r2 = vv[t][2][w], r3 = vv[t][3][w];
                const u32x2 even = {(r0 & 0xffffu) | (r1 << 16), (r2 & 0xffffu) | (r3 << 16)};
                const u32x2 odd = {(r0 >> 16) | (r1 & 0xffff0000u), (r2 >> 16) | (r3 & 0xffff0000u)};
                O[t][2 * w] = Mma<T>::pv(p_hi, even, O[t][2 * w]);
                O[t][2 * w] = Mma<T>::pv(p_lo, even, O[t][2 * w]);
                O[t][2 * w + 1] = Mma<T>::pv(p_hi, odd, O[t][2 * w + 1]);
                O[t][2 * w + 1] = Mma<T>::pv(p_lo, odd, O[t][2 * w + 1]);
            }
        }
    };

    for (int run = 0; run < 4; ++run) {
        int lo, hi, phys0;
        run_bounds(a, x, run, lo, hi, phys0);
        if (hi - lo <= 0) continue;
        const char *kp, *vp;
        const int lead = phys0 & (WROWS - 1);             // rows between the aligned anchor and the run's first row
        const int cnt = hi - lo + lead;                   // run length measured from the anchor
        if (run < 3) {
            kp = Kb + (size_t)phys0 * ROWB;
            vp = Vb + (size_t)phys0 * ROWB;
        } else {                                          // eq. 2: the new row comes from the caller and joins the cache
            kp = (const char*)a.k_new + (size_t)unit * ROWB;
            vp = (const char*)a.v_new + (size_t)unit * ROWB;
            if (tid < NCH) {
                *(u32x4*)(Kb + (size_t)a.new_phys * ROWB + tid * 16) = *(const u32x4*)(kp + tid * 16);
                *(u32x4*)(Vb + (size_t)a.new_phys * ROWB + tid * 16) = *(const u32x4*)(vp + tid * 16);
                if (tid == 0) a.pos[x.ubase + a.new_phys] = a.new_pos;
            }
        }
        for (int base = wave * WROWS; base < cnt; base += NW * WROWS) {   // waves take tiles round-robin
            u32x4 kk[QP], vv[VS][4];                      // (double-buffering was measured 4% slower here)
            load_tile(kk, vv, kp, vp, base, lead, cnt);
            compute_tile(kk, vv, base, lead, cnt, lo - j0 + base - lead);
        }
    }

    // this wave's result into LDS in the layout finish_split expects
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (q == 0 && j < G) { sm_m[wave][j] = m_run; sm_l[wave][j] = l_tot; }
#pragma unroll
    for (int t = 0; t < VS; ++t) {
        if (16 * t + j < NCH) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int head = 4 * q + v;
                if (head < G) {
#pragma unroll
                    for (int mcol = 0; mcol < 8; ++mcol) sm_acc[wave][head][8 * (16 * t + j) + mcol] = O[t][mcol][v];
                }
            }
        }
    }
    finish_split<G, D, NW>(a, x, stage, sm_m, sm_l, sm_acc, sm_ml, &sm_ticket);
}

constexpr int kScoreRowsPerBlock = 2048;

// Applies the pending score update of the last decode step to every retained row right away.
template <int G>
__global__ __launch_bounds__(256) void flush_scores_kernel(const AttnArgs a)
{
    const int chunk = blockIdx.x, unit = blockIdx.y, tid = threadIdx.x;
    float M[G], iL[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        M[g] = a.stat_prev[((size_t)unit * G + g) * 2];
        iL[g] = a.stat_prev[((size_t)unit * G + g) * 2 + 1];
    }
    const size_t ubase = (size_t)unit * a.cap;
    const float* logit_u = a.logit_prev + ubase * G;
    const int jbeg = chunk * kScoreRowsPerBlock;
    const int jend = min(a.n, jbeg + kScoreRowsPerBlock);
    for (int j = jbeg + tid; j < jend; j += 256) {
        const int ph = a.map.phys(j);
        float sc = a.score[ubase + ph];
#pragma unroll
        for (int g = 0; g < G; ++g) sc += fast_exp2(logit_u[(size_t)g * a.cap + ph] - M[g]) * iL[g];
        a.score[ubase + ph] = sc;
    }
}

template <int G> constexpr int unroll_for() { return G == 1 ? BUZZ_U_G1 : (G == 2 ? BUZZ_U_G2 : (G == 4 ? BUZZ_U_G4 : BUZZ_U_G8)); }

template <typename T, int D, int G>
hipError_t launch_split_t(const AttnArgs& a, int units, hipStream_t st, Timing tm)
{
    dim3 grid(a.n_splits, units), block(a.waves * 64);
    const size_t lds = (size_t)G * a.rows_per_split * sizeof(float);   // logit staging
    if constexpr (G >= 2 && !std::is_same<T, float>::value) {   // grouped queries on a 16-bit cache: matrix cores
        if (a.waves == 8) {
            if (a.streaming) BUZZ_LAUNCH((attn_split_mfma_kernel<T, D, G, true, 8>), grid, block, lds, st, tm, a);
            else BUZZ_LAUNCH((attn_split_mfma_kernel<T, D, G, false, 8>), grid, block, lds, st, tm, a);
        } else {
            if (a.streaming) BUZZ_LAUNCH((attn_split_mfma_kernel<T, D, G, true, 4>), grid, block, lds, st, tm, a);
            else BUZZ_LAUNCH((attn_split_mfma_kernel<T, D, G, false, 4>), grid, block, lds, st, tm, a);
        }
        return hipGetLastError();
    }
    constexpr int RPW = 64 / (D / Elem<T>::VEC);
    constexpr int U = unroll_for<G>() * RPW >= 4 ? unroll_for<G>() : 4 / RPW;   // a trip covers at least 4 rows
    if (a.waves == 8) {
        if (a.streaming) BUZZ_LAUNCH((attn_split_kernel<T, D, G, U, true, 8>), grid, block, lds, st, tm, a);
        else BUZZ_LAUNCH((attn_split_kernel<T, D, G, U, false, 8>), grid, block, lds, st, tm, a);
    } else {
        if (a.streaming) BUZZ_LAUNCH((attn_split_kernel<T, D, G, U, true, 4>), grid, block, lds, st, tm, a);
        else BUZZ_LAUNCH((attn_split_kernel<T, D, G, U, false, 4>), grid, block, lds, st, tm, a);
    }
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_split_g(int G, const AttnArgs& a, int units, hipStream_t st, Timing tm)
{
    switch (G) {
        case 1: return launch_split_t<T, D, 1>(a, units, st, tm);
        case 2: return launch_split_t<T, D, 2>(a, units, st, tm);
        case 4: return launch_split_t<T, D, 4>(a, units, st, tm);
        case 8: return launch_split_t<T, D, 8>(a, units, st, tm);
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_split_d(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm)
{
    switch (D) {
        case 64: return launch_split_g<T, 64>(G, a, units, st, tm);
        case 128: return launch_split_g<T, 128>(G, a, units, st, tm);
        case 256: return launch_split_g<T, 256>(G, a, units, st, tm);
    }
    return hipErrorInvalidValue;
}

}  // namespace

// This file is compiled four times (BUZZ_TU = 0, 1, 2: the streaming kernels of one dtype each;
// BUZZ_TU = 3: everything that does not depend on the dtype), so that the build runs in parallel.
#ifndef BUZZ_TU
#error "compile with -DBUZZ_TU=0..3 (see build.py)"
#endif
#if BUZZ_TU == 0
hipError_t launch_attn_split_fp32(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm) { return launch_split_d<float>(D, G, a, units, st, tm); }
#elif BUZZ_TU == 1
hipError_t launch_attn_split_fp16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm) { return launch_split_d<fp16_t>(D, G, a, units, st, tm); }
#elif BUZZ_TU == 2
hipError_t launch_attn_split_bf16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm) { return launch_split_d<bf16_t>(D, G, a, units, st, tm); }
#else
hipError_t launch_attn_split_fp32(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm);
hipError_t launch_attn_split_fp16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm);
hipError_t launch_attn_split_bf16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm);

bool attn_supported(int dtype, int D, int G)
{
    if (dtype != BUZZ_FP32 && dtype != BUZZ_FP16 && dtype != BUZZ_BF16) return false;
    if (D != 64 && D != 128 && D != 256) return false;
    return G == 1 || G == 2 || G == 4 || G == 8;
}

int attn_tile_rows(int dtype, int D, int G)
{
    const int vec = dtype == BUZZ_FP32 ? 4 : 8;
    const int rpw = 64 / (D / vec);
    if (G >= 2 && dtype != BUZZ_FP32) return 4 * 16;      // matrix-core kernel: 16-row tiles
    int u = G == 1 ? BUZZ_U_G1 : (G == 2 ? BUZZ_U_G2 : (G == 4 ? BUZZ_U_G4 : BUZZ_U_G8));
    if (u * rpw < 4) u = 4 / rpw;
    return 4 * rpw * u;
}

hipError_t launch_attn_split(int dtype, int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm)
{
    switch (dtype) {
        case BUZZ_FP32: return launch_attn_split_fp32(D, G, a, units, st, tm);
        case BUZZ_FP16: return launch_attn_split_fp16(D, G, a, units, st, tm);
        case BUZZ_BF16: return launch_attn_split_bf16(D, G, a, units, st, tm);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_flush_scores(int G, const AttnArgs& a, int units, hipStream_t st, Timing tm)
{
    if (a.n <= 0) return hipSuccess;
    dim3 grid((a.n + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock, units), block(256);
    switch (G) {
        case 1: BUZZ_LAUNCH((flush_scores_kernel<1>), grid, block, 0, st, tm, a); break;
        case 2: BUZZ_LAUNCH((flush_scores_kernel<2>), grid, block, 0, st, tm, a); break;
        case 4: BUZZ_LAUNCH((flush_scores_kernel<4>), grid, block, 0, st, tm, a); break;
        case 8: BUZZ_LAUNCH((flush_scores_kernel<8>), grid, block, 0, st, tm, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
#endif  // BUZZ_TU

}  // namespace buzz
