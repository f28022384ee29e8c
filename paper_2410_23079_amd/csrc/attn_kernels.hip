// Decode attention over the retained BUZZ cache (eq. 3 / eq. 5 of the paper) as ONE kernel per step:
// the append of eq. 2, the split-softmax attention, the merge of the splits and the accumulated-score
// update ("A" of Alg. 2) all happen inside attn_split.
//
//  - One block per (key-range split, unit).  Two streaming variants: on the vector ALU a wave reads
//    64 x 16 B per load instruction = RPW consecutive cache rows, LPR = 64 / RPW lanes per row (every
//    load is one contiguous 1 KB burst), q.k is a two-element-dot chain per lane plus an LPR-lane DPP
//    reduction, softmax runs online per lane group and p.V accumulates in registers; with several
//    query heads per kv head on a 16-bit cache both contractions run on the matrix cores instead.
//  - The scaled logit of every row is written to a scratch array.  A row's probability needs the
//    maximum and sum over ALL splits, which only exist once the step is over, so the score update of
//    step t is applied by step t+1 while it streams the same rows anyway (one lane per row, coalesced):
//    score += sum_g exp2(logit_t - M_t[g]) / L_t[g].  flush_scores applies a pending update to every row
//    right away (before an export, or an eviction that moves old rows); the usual eviction applies it only to
//    the rows it ranks and leaves the rest pending.
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
// 16-byte loads of K (and of V) per lane and tile.  Group size 1 keeps two tiles in flight; small tiles win
// there because the waves claim them dynamically (finer balance): 2 loads when the cache streams from HBM
// (4: -2%, 1: -9%, too little in flight), 1 load when it is served by the last-level cache (+3.5% over 2).
#ifndef BUZZ_U_G1
#define BUZZ_U_G1 2
#endif
#ifndef BUZZ_U_G1_CACHED
#define BUZZ_U_G1_CACHED 1
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
#ifndef BUZZ_MFMA_TR
#define BUZZ_MFMA_TR 1   // 16-row tiles a wave of the matrix-core kernel has in flight
#endif
#ifndef BUZZ_MIN_BLOCKS
#define BUZZ_MIN_BLOCKS 1  // second argument of __launch_bounds__
#endif

// Optional in-kernel time stamps (a tuning aid, compiled out unless BUZZ_TRACE is defined): slot s of
// block b holds the wall clock (100 MHz) at which the block passed point s of the last launch.
#if defined(BUZZ_TRACE) && BUZZ_TU == 2
__device__ unsigned long long g_trace[kMaxBlocks * 16];
#define BUZZ_STAMP(slot) do { g_trace[(size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 16 + (slot)] = wall_clock64(); } while (0)
#define BUZZ_STAMP_VALUE(slot, v) do { g_trace[(size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 16 + (slot)] = (v); } while (0)
#else
#define BUZZ_STAMP(slot) do { } while (0)
#define BUZZ_STAMP_VALUE(slot, v) do { } while (0)
#endif

template <typename T> struct Elem;
// cvt: 16 bytes -> VEC floats.  dot: sum over the 16 bytes of q * k in fp32 (16-bit types use the
// two-element dot instruction on the raw words: exact products, fp32 accumulation, no conversion).
template <> struct Elem<float> {
    [[maybe_unused]] static constexpr int VEC = 4;
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
    [[maybe_unused]] static constexpr int VEC = 8;
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
    [[maybe_unused]] static constexpr int VEC = 8;
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

// How split partials travel between the blocks of one launch (finish_split_scoped).
//
// Device-wide form (blocks of a unit possibly on different dies, each die with its own L2).  A block writes
// its partial with relaxed device-scope atomic stores (`sc1`: written through the die's L2 to the memory
// side), every wave waits with s_waitcnt vmcnt(0) for its own stores, the block synchronises, one thread takes
// a ticket (relaxed atomic add), and the block that draws the last ticket reads every partial with relaxed
// device-scope atomic loads (`sc1`: not served from a die's private copy).  Why the merging block cannot see a
// stale partial: this is the compiler's own release / acquire sequence for device scope on this target with
// the two cache-wide operations taken out, and neither is needed here.
//   * Release side.  The documented release sequence is "write back the L2 (buffer_wbl2 sc1), then
//     s_waitcnt vmcnt(0), then the releasing atomic".  vmcnt counts a store until the level that the store's
//     scope names has acknowledged it; that is what makes the wait the completion point of the sequence, and
//     for an sc1 store the acknowledgement comes from the memory side.  The write-back exists for data written
//     earlier with weaker scope that may still sit dirty in the L2; every byte of a partial is written with an
//     sc1 store, so there is nothing to write back.  (A device-scope fence here costs a full L2 write-back per
//     block: 2.5-30x on the whole kernel.)  The wait is per wave, so every wave executes it before the block
//     barrier, and only after the barrier does thread 0 take the ticket: the ticket is ordered after the
//     acknowledgement of every store of the block.  Without the explicit wait the compiler is free to let the
//     relaxed stores drain later, and the ticket then overtook a partial about once in 10^5 launches.
//   * Acquire side.  The documented acquire sequence is "the acquiring atomic, then invalidate L1 and the
//     non-local L2 lines (buffer_inv sc1)", so that LATER ORDINARY loads cannot hit stale copies.  The merging
//     block reads the partials with sc1 atomic loads, which are coherent at device scope by themselves, so no
//     invalidate is needed.  They cannot start early: the ticket's value goes through LDS and a block barrier
//     to every thread, the loads are control-dependent on it (`last`), and a workgroup-scope acquire fence
//     sits between the barrier and the loads, across which the compiler may not move atomic accesses.
//   * The ticket itself is one atomic counter per unit; read-modify-write atomics execute at the point of
//     coherence of their address whatever cache holds a copy.  The merging block resets it for the next launch.
// Nobody waits for anybody: a block that is not last simply ends.
//
// Die-local form (LOCAL = true).  When all blocks of a unit run on ONE die (the host arranges that by block
// number where the shape allows, see make_ctx), the same handshake runs one level lower: workgroup-scope
// atomic stores and loads (`sc0`: through the compute unit's L1, served by the die's L2, which all its compute
// units share), the same wait, the same ticket.  The hardware argument is the same with "the die's L2" in
// place of "the memory side".  It lies outside the language memory model, which knows no scope between one
// workgroup and the device, so it is guarded twice: the host enables it only on a GPU where a probe launch
// has shown that block numbers equal mod 8 share a die, and every block compares the die it actually runs on
// with the probe's record and flags a difference in the ticket, which turns the unit's output into NaN.
// BUZZ_FLAG_DEVICE_MERGE selects the device-wide form everywhere.
template <bool LOCAL> constexpr int merge_scope() { return LOCAL ? __HIP_MEMORY_SCOPE_WORKGROUP : __HIP_MEMORY_SCOPE_AGENT; }
template <bool LOCAL> __device__ inline void publish(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, merge_scope<LOCAL>()); }
template <bool LOCAL> __device__ inline float acquire(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, merge_scope<LOCAL>()); }

// Where a block works: logical rows [j0, j1) of one unit.  The range is cut into at most four physically
// contiguous runs (linear region, ring before the wrap, ring after the wrap, the row being appended).
struct SplitCtx {
    int split, unit, b, kvh;
    int home;            // die-local merge: launch-order block number mod 8, which decides the die
    int j0, j1, jl1, wrap;
    size_t ubase;
};

__device__ inline SplitCtx make_ctx(const AttnArgs& a)
{
    SplitCtx x;
    x.split = blockIdx.x; x.unit = blockIdx.y;
    x.home = 0;
    if (a.xcd_local) {
        // The hardware deals the blocks of a grid to the dies (XCDs) round-robin in launch order: block b runs
        // on die b mod 8.  Renumber so that the n_splits blocks of a unit share b mod 8 (units is a multiple of
        // 8 here): die d gets units d * units/8 ... and, in launch order, their splits.
        const int b = blockIdx.y * gridDim.x + blockIdx.x, die = b & 7, slot = b >> 3;
        x.unit = die * (gridDim.y >> 3) + slot / (int)gridDim.x;
        x.split = slot % (int)gridDim.x;
        x.home = die;
    }
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
    else { lo = a.n - 1; hi = (x.j1 == a.n && x.j0 < a.n) ? a.n : lo; phys0 = a.new_phys; }
}

// Everything a block does once its waves have put their (max, sum, unnormalised output) into LDS.
// The order hides as much latency as it can behind work that does not depend on it:
//   2. merge the waves, publish the split's partial (write-through stores);
//   3. wait for the published stores, synchronise, take the ticket;
//   4. the block that drew the last ticket requests the partials (upper half of its waves);
//   5. side phase: this step's logits leave LDS, the previous step's score update is applied
//      (off the critical path: in the last block it runs under the latency of step 4's loads);
//   6. the last block merges the splits and writes the output.
// The tiles of a split, numbered across its (up to three) stored runs.  Inside a run tiles sit on a grid
// anchored at a physical multiple of WROWS: `lead` rows before the run's first row are masked, `cnt` is
// the run length measured from the anchor.  A block's waves do not own fixed tiles: apart from the first
// one each, a wave claims its next tile from a counter in LDS when it has issued the loads of the current
// one.  (With fixed round-robin tiles the waves launched first -- which the memory pipeline serves first
// -- ended 15% earlier than the others, and the block waited for the slowest.)
template <int WROWS>
struct TileMap {
    int lo0, lo1, lo2, ph0, ph1, ph2, ld0, ld1, ld2, c0, c1, c2, f1, f2, n_tiles;
    __device__ inline TileMap(const AttnArgs& a, const SplitCtx& x)
    {
        int h;
        run_bounds(a, x, 0, lo0, h, ph0); ld0 = ph0 & (WROWS - 1); c0 = h > lo0 ? h - lo0 + ld0 : 0;
        run_bounds(a, x, 1, lo1, h, ph1); ld1 = ph1 & (WROWS - 1); c1 = h > lo1 ? h - lo1 + ld1 : 0;
        run_bounds(a, x, 2, lo2, h, ph2); ld2 = ph2 & (WROWS - 1); c2 = h > lo2 ? h - lo2 + ld2 : 0;
        f1 = (c0 + WROWS - 1) / WROWS;
        f2 = f1 + (c1 + WROWS - 1) / WROWS;
        n_tiles = f2 + (c2 + WROWS - 1) / WROWS;
    }
    __device__ inline int total() const { return n_tiles; }
    // tile t -> its run's (lo, phys0, lead, cnt) and the tile's first row measured from the anchor
    __device__ inline void locate(int t, int& l, int& p, int& ld, int& c, int& base) const
    {
        // (sums of "difference or 0" rather than nested selects between members: the latter turn into
        // an indexed read of the structure and push it into private memory)
        const bool r1 = t >= f1, r2 = t >= f2;
        l = lo0 + (r1 ? lo1 - lo0 : 0) + (r2 ? lo2 - lo1 : 0);
        p = ph0 + (r1 ? ph1 - ph0 : 0) + (r2 ? ph2 - ph1 : 0);
        ld = ld0 + (r1 ? ld1 - ld0 : 0) + (r2 ? ld2 - ld1 : 0);
        c = c0 + (r1 ? c1 - c0 : 0) + (r2 ? c2 - c1 : 0);
        base = (t - (r1 ? f1 : 0) - (r2 ? f2 - f1 : 0)) * WROWS;
    }
};

__device__ inline int claim_tile(int* counter)
{
    int t = 0;
    if ((threadIdx.x & 63) == 0) t = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return __builtin_amdgcn_readfirstlane(t);
}

// The tile a wave takes after tile `last`: claimed from the block's counter, or -- when the caller asked
// for results that do not depend on timing -- the next one of a fixed round-robin over `nw` waves.
__device__ inline int next_tile(const AttnArgs& a, int* counter, int last, int nw)
{
    return a.fixed_tiles ? last + nw : claim_tile(counter);
}

// The previous step's softmax statistics of one unit (global maximum and 1/sum per head), which turn its
// stored logits into probabilities.  A kernel requests them when it starts: they come from memory, and a
// request made where they are needed would stall the end of the block for a full round trip.
template <int G> struct PrevStat { float M[G], iL[G]; };

template <int G>
__device__ inline PrevStat<G> load_prev_stat(const AttnArgs& a, int unit)
{
    PrevStat<G> p;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        p.M[g] = a.pending ? a.stat_prev[((size_t)unit * G + g) * 2] : 0.f;
        p.iL[g] = a.pending ? a.stat_prev[((size_t)unit * G + g) * 2 + 1] : 0.f;
    }
    return p;
}

// What a thread needs for the first pass of its side phase (4 consecutive physical rows in each stored
// run of the split): the old scores and the previous step's logits.  Requested when the kernel starts and
// consumed after the streaming loop, so that their latency is never exposed.
// (They occupy 12 (G + 1) registers through the whole streaming loop; where that would spill -- 8 heads
// per row, or 4 heads of 256 columns -- the request is made after the loop instead.)
template <int G> struct SideRows { float4 sc[3], lp[3][G]; };
template <int G, int D> constexpr bool early_side() { return G <= 4 && G * D <= 512; }

template <int G>
__device__ inline void request_side_rows(const AttnArgs& a, const SplitCtx& x, SideRows<G>& p)
{
    const int tid = threadIdx.x;
    const float* logit_prev_u = a.logit_prev + x.ubase * G;
    const float* score_u = a.score + x.ubase;
#pragma unroll
    for (int run = 0; run < 3; ++run) {
        int lo, hi, phys0;
        run_bounds(a, x, run, lo, hi, phys0);
        const int lead = phys0 & 3, pa = phys0 - lead, cnt = hi - lo + lead;
        if (a.pending && hi - lo > 0 && 4 * tid < cnt) {
            p.sc[run] = *(const float4*)(score_u + pa + 4 * tid);
#pragma unroll
            for (int g = 0; g < G; ++g) p.lp[run][g] = *(const float4*)(logit_prev_u + (size_t)g * a.cap + pa + 4 * tid);
        }
    }
}

// new score = old score + sum over heads of the previous step's probability (lazy update, one step late)
template <int G>
__device__ inline void first_pass_scores(const AttnArgs& a, const SplitCtx& x, const PrevStat<G>& prev, SideRows<G>& p)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int run = 0; run < 3; ++run) {
        int lo, hi, phys0;
        run_bounds(a, x, run, lo, hi, phys0);
        const int lead = phys0 & 3, cnt = hi - lo + lead;
        if (a.pending && hi - lo > 0 && 4 * tid < cnt) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                p.sc[run].x = add_probability(p.sc[run].x, p.lp[run][g].x, prev.M[g], prev.iL[g]);
                p.sc[run].y = add_probability(p.sc[run].y, p.lp[run][g].y, prev.M[g], prev.iL[g]);
                p.sc[run].z = add_probability(p.sc[run].z, p.lp[run][g].z, prev.M[g], prev.iL[g]);
                p.sc[run].w = add_probability(p.sc[run].w, p.lp[run][g].w, prev.M[g], prev.iL[g]);
            }
        }
    }
}

template <int G, int D, int NW, bool LOCAL>
__device__ inline void finish_split_scoped(const AttnArgs& a, const SplitCtx& x, const PrevStat<G>& prev,
                                    const float4 (&pre_sc)[3], const float* stage,
                                    float (*sm_m)[G], float (*sm_l)[G], float (*sm_acc)[G][D], int* sm_ticket)
{
    constexpr int NTHR = NW * 64;                         // threads per block
    const int tid = threadIdx.x;
    const int unit = x.unit, j0 = x.j0;
    const int S = a.n_splits;
    float* logit_u = a.logit + x.ubase * G;               // [G][cap] for this unit, written by this step
    const float* logit_prev_u = a.logit_prev + x.ubase * G;   // the previous step's logits
    float* score_u = a.score + x.ubase;
    const float (&Mp)[G] = prev.M;
    const float (&iLp)[G] = prev.iL;

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
            publish<LOCAL>(a.part_o + (pbase + g) * D + d, o);
            if (d == 0) {
                publish<LOCAL>(a.part_ml + (pbase + g) * 2, M);
                publish<LOCAL>(a.part_ml + (pbase + g) * 2 + 1, L);
            }
        }
    }

    if (tid == 0) BUZZ_STAMP(2);

    // 3. ticket: the block that arrives last for this unit sees every split's partial.  Every wave first
    // waits until its own published stores have been acknowledged (vmcnt(0)), then the block synchronises,
    // then one thread takes the ticket: the ticket can never overtake a partial (the argument is written out
    // above merge_scope).  No cache maintenance is involved.
    bool last = false;
    if (S > 1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0), expcnt / lgkmcnt untouched
        __syncthreads();
        if (tid == 0) {
            // A die-local merge is only right if this block really runs where its number says: the host has
            // recorded which die served block numbers 0..7 (die_map, 4 bits each); a block that finds itself
            // elsewhere says so in the ticket's upper half, and the merging block sees every earlier arrival's.
            int add = 1;
            if (LOCAL && (__builtin_amdgcn_s_getreg((31 << 11) | 20) & 7u) != ((a.die_map >> (4 * x.home)) & 15u)) add += 0x10000;   // XCC_ID
            const int before = __hip_atomic_fetch_add(a.ticket + unit, add, __ATOMIC_RELAXED, merge_scope<LOCAL>());
            *sm_ticket = before + (add & 0x10000);
        }
        __syncthreads();
        last = (*sm_ticket & 0xffff) == S - 1;
        if (tid == 0) BUZZ_STAMP(4);
    }

    // 4. in the last block the upper half of the waves merges the splits; each of those threads owns OPT
    // output elements and requests, for the first CH splits, the element itself and the (max, sum) pair of
    // its head -- everything in ONE round of device-scope loads with no branch in between.  The answers
    // arrive while the block does its side phase, which for up to 4 * NTHR / 2 rows per split keeps only
    // the lower half of the waves busy.
    constexpr int NM = NTHR / 2;                          // merging threads
    constexpr int OPT = (G * D + NM - 1) / NM;            // output elements per merging thread
    constexpr int CH = OPT >= 16 ? 2 : (OPT >= 8 ? 4 : 8);   // splits per round of loads
    const bool merger = last && tid >= NM;
    const unsigned long long* ml = (const unsigned long long*)(a.part_ml + (size_t)unit * a.s_cap * G * 2);
    const float* po = a.part_o + (size_t)unit * a.s_cap * G * D;
    unsigned long long mlr[OPT][CH];
    float xr[OPT][CH];
    auto request = [&](int s0) {
#pragma unroll
        for (int r = 0; r < OPT; ++r) {
            const int i = min(tid - NM + NM * r, G * D - 1);
            const int g = i / D;
#pragma unroll
            for (int e = 0; e < CH; ++e) {
                const int sp = min(s0 + e, S - 1);
                mlr[r][e] = __hip_atomic_load(ml + sp * G + g, __ATOMIC_RELAXED, merge_scope<LOCAL>());
                xr[r][e] = acquire<LOCAL>(po + (size_t)sp * G * D + i);
            }
        }
    };
    if (last) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (merger) request(0);

    // 5. dense side phase, after the read stream of this block is over (the logits staged by all waves are
    // visible after the barriers above).  Four consecutive physical rows per thread, 16-byte accesses where
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
                if (run < 3 && r0 == 4 * tid) {           // first pass: worked out in step 2b
                    sc = pre_sc[run < 3 ? run : 0];
                } else {
                    float4 lp[G];
                    sc = *(const float4*)(score_u + ph);
#pragma unroll
                    for (int g = 0; g < G; ++g) lp[g] = *(const float4*)(logit_prev_u + (size_t)g * a.cap + ph);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        sc.x = add_probability(sc.x, lp[g].x, Mp[g], iLp[g]);
                        sc.y = add_probability(sc.y, lp[g].y, Mp[g], iLp[g]);
                        sc.z = add_probability(sc.z, lp[g].z, Mp[g], iLp[g]);
                        sc.w = add_probability(sc.w, lp[g].w, Mp[g], iLp[g]);
                    }
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
    if (tid == 0) BUZZ_STAMP(3);
    if (!merger) return;

    // 6. merge the splits: a running (max, sum, output) per owned element, CH splits per round.
    // A die-local merge with a block on an unexpected die may have missed partials: its output is NaN rather
    // than plausible numbers.
    const float poison = (*sm_ticket >> 16) ? __builtin_nanf("") : 0.f;
    float Mr[OPT], Lr[OPT], Or[OPT];
#pragma unroll
    for (int r = 0; r < OPT; ++r) { Mr[r] = -INFINITY; Lr[r] = 0.f; Or[r] = 0.f; }
    for (int s0 = 0; s0 < S; s0 += CH) {
        if (s0 > 0) request(s0);
#pragma unroll
        for (int r = 0; r < OPT; ++r) {
            float mx = Mr[r];
#pragma unroll
            for (int e = 0; e < CH; ++e)
                if (s0 + e < S) mx = fmaxf(mx, __uint_as_float((unsigned)mlr[r][e]));   // finite: the appended row is always present
            const float keep = fast_exp2(Mr[r] - mx);    // 0 in the first round
            Lr[r] *= keep; Or[r] *= keep; Mr[r] = mx;
#pragma unroll
            for (int e = 0; e < CH; ++e) {
                if (s0 + e < S) {
                    const float w = fast_exp2(__uint_as_float((unsigned)mlr[r][e]) - mx);
                    Lr[r] = fmaf(__uint_as_float((unsigned)(mlr[r][e] >> 32)), w, Lr[r]);
                    Or[r] = fmaf(w, xr[r][e], Or[r]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < OPT; ++r) {
        const int i = tid - NM + NM * r;
        if (i >= G * D) continue;
        const int g = i / D;
        outp[i] = Or[r] / Lr[r] + poison;
        if (i - g * D == 0) {
            a.stat[((size_t)unit * G + g) * 2] = Mr[r];
            a.stat[((size_t)unit * G + g) * 2 + 1] = 1.0f / Lr[r];
        }
    }
    if (tid == NM) __hip_atomic_store(a.ticket + unit, 0, __ATOMIC_RELAXED, merge_scope<LOCAL>());   // ready for the next step
    if (tid == NM) BUZZ_STAMP(5);
}

template <int G, int D, int NW>
__device__ inline void finish_split(const AttnArgs& a, const SplitCtx& x, const PrevStat<G>& prev,
                                    const float4 (&pre_sc)[3], const float* stage,
                                    float (*sm_m)[G], float (*sm_l)[G], float (*sm_acc)[G][D], int* sm_ticket)
{
    if (a.xcd_local) finish_split_scoped<G, D, NW, true>(a, x, prev, pre_sc, stage, sm_m, sm_l, sm_acc, sm_ticket);
    else finish_split_scoped<G, D, NW, false>(a, x, prev, pre_sc, stage, sm_m, sm_l, sm_acc, sm_ticket);
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
    __shared__ int sm_ticket, sm_next;

    const SplitCtx x = make_ctx(a);
    const int unit = x.unit, b = x.b, kvh = x.kvh, j0 = x.j0, j1 = x.j1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane % LPR, rs = lane / LPR;
    const PrevStat<G> prev = load_prev_stat<G>(a, unit);
    SideRows<G> side;
    if constexpr (early_side<G, D>()) request_side_rows<G>(a, x, side);
    if (tid == 0) { BUZZ_STAMP(0); BUZZ_STAMP_VALUE(6, __builtin_amdgcn_s_getreg((31 << 11) | 4)); BUZZ_STAMP_VALUE(7, __builtin_amdgcn_s_getreg((31 << 11) | 20)); }

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
    // contiguous runs; inside a run, tiles of WROWS rows sit on a grid anchored at a physical multiple
    // of WROWS (`lead` rows before the run's first row are masked), and the block's waves take the tiles
    // of all runs one after another (TileMap).  The streaming phase only reads: logits are staged in LDS,
    // and all per-row side traffic (this step's logits out, the previous step's logits and the old score
    // in, the new score out) happens in one dense phase at the end of the block.  Writes that trickle
    // into a saturated read stream were measured to cost ~5% of the kernel per 1% of extra bytes.
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

    if (tid == 0) sm_next = NW;                           // tiles 0 .. NW-1 are the waves' first tiles
    __syncthreads();

    // eq. 2: the new row comes from the caller, joins the cache, and is attended to like any other row
    if (x.j1 == a.n && x.j0 < a.n && wave == 0) {
        const char* kp = (const char*)a.k_new + (size_t)unit * ROWB;
        const char* vp = (const char*)a.v_new + (size_t)unit * ROWB;
        if (rs == 0) {
            *(u32x4*)(Kb + (size_t)a.new_phys * ROWB + lane_off) = *(const u32x4*)(kp + lane_off);
            *(u32x4*)(Vb + (size_t)a.new_phys * ROWB + lane_off) = *(const u32x4*)(vp + lane_off);
            if (c == 0) a.pos[ubase + a.new_phys] = a.new_pos;
        }
        u32x4 kr[U], vr[U];
        load_tile(kr, vr, kp, vp, 0, 0, 1);
        compute_tile(kr, vr, 0, 0, 1, a.n - 1 - j0);
    }

    const TileMap<WROWS> tiles(a, x);
    const int total = tiles.total();
    auto load_t = [&](u32x4 (&kr)[U], u32x4 (&vr)[U], int t) {
        int lo, phys0, lead, cnt, base;
        tiles.locate(t, lo, phys0, lead, cnt, base);
        load_tile(kr, vr, Kb + (size_t)phys0 * ROWB, Vb + (size_t)phys0 * ROWB, base, lead, cnt);
    };
    auto compute_t = [&](const u32x4 (&kr)[U], const u32x4 (&vr)[U], int t) {
        int lo, phys0, lead, cnt, base;
        tiles.locate(t, lo, phys0, lead, cnt, base);
        compute_tile(kr, vr, base, lead, cnt, lo - j0 + base - lead);
    };
    if constexpr (G == 1) {
        // two tile buffers: the next tile's loads are issued before the current tile is consumed
        u32x4 ka[U], va[U], kb[U], vb[U];
        int t = wave, tn = next_tile(a, &sm_next, t, NW);
        if (t < total) load_t(ka, va, t);
        while (t < total) {
            if (tn < total) load_t(kb, vb, tn);
            int tnn = next_tile(a, &sm_next, tn, NW);
            compute_t(ka, va, t);
            t = tn; tn = tnn;
            if (t >= total) break;
            if (tn < total) load_t(ka, va, tn);
            tnn = next_tile(a, &sm_next, tn, NW);
            compute_t(kb, vb, t);
            t = tn; tn = tnn;
        }
    } else {
        int t = wave;
        while (t < total) {
            u32x4 kr[U], vr[U];
            load_t(kr, vr, t);
            const int tn = next_tile(a, &sm_next, t, NW);
            compute_t(kr, vr, t);
            t = tn;
        }
    }

    if (lane == 0) BUZZ_STAMP(8 + (wave & 7));
    if constexpr (!early_side<G, D>()) request_side_rows<G>(a, x, side);
    first_pass_scores<G>(a, x, prev, side);

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
    finish_split<G, D, NW>(a, x, prev, side.sc, stage, sm_m, sm_l, sm_acc, &sm_ticket);
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
    constexpr int TR = BUZZ_MFMA_TR;                      // tiles a wave loads before it computes
    static_assert(G >= 2 && G <= 16 && NCH % 4 == 0, "grouped queries, head_dim multiple of 32");

    extern __shared__ float stage[];                      // [G][rows_per_split] logits of this split's rows
    __shared__ float sm_m[NW][G], sm_l[NW][G];
    __shared__ float sm_acc[NW][G][D];
    __shared__ int sm_ticket, sm_next;

    const SplitCtx x = make_ctx(a);
    const int unit = x.unit, j0 = x.j0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;
    const PrevStat<G> prev = load_prev_stat<G>(a, unit);
    SideRows<G> side;
    if constexpr (early_side<G, D>()) request_side_rows<G>(a, x, side);
    if (tid == 0) { BUZZ_STAMP(0); BUZZ_STAMP_VALUE(6, __builtin_amdgcn_s_getreg((31 << 11) | 4)); BUZZ_STAMP_VALUE(7, __builtin_amdgcn_s_getreg((31 << 11) | 20)); }

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

    if (tid == 0) sm_next = NW;                           // tiles 0 .. NW-1 are the waves' first tiles
    __syncthreads();

    // eq. 2: the new row comes from the caller, joins the cache, and is attended to like any other row
    if (x.j1 == a.n && x.j0 < a.n && wave == 0) {
        const char* kp = (const char*)a.k_new + (size_t)unit * ROWB;
        const char* vp = (const char*)a.v_new + (size_t)unit * ROWB;
        if (tid < NCH) {
            *(u32x4*)(Kb + (size_t)a.new_phys * ROWB + tid * 16) = *(const u32x4*)(kp + tid * 16);
            *(u32x4*)(Vb + (size_t)a.new_phys * ROWB + tid * 16) = *(const u32x4*)(vp + tid * 16);
            if (tid == 0) a.pos[x.ubase + a.new_phys] = a.new_pos;
        }
        u32x4 kk[QP], vv[VS][4];
        load_tile(kk, vv, kp, vp, 0, 0, 1);
        compute_tile(kk, vv, 0, 0, 1, a.n - 1 - j0);
    }

    // groups of TR tiles: all loads of a group are in flight before its first tile is used
    const TileMap<WROWS * TR> tiles(a, x);
    const int total = tiles.total();
    int t = wave;
    while (t < total) {
        int lo, phys0, lead, cnt, base;
        tiles.locate(t, lo, phys0, lead, cnt, base);
        const char* kp = Kb + (size_t)phys0 * ROWB;
        const char* vp = Vb + (size_t)phys0 * ROWB;
        u32x4 kk[TR][QP], vv[TR][VS][4];
#pragma unroll
        for (int u = 0; u < TR; ++u)
            if (u == 0 || base + u * WROWS < cnt) load_tile(kk[u], vv[u], kp, vp, base + u * WROWS, lead, cnt);
        const int tn = next_tile(a, &sm_next, t, NW);
#pragma unroll
        for (int u = 0; u < TR; ++u)
            if (u == 0 || base + u * WROWS < cnt)
                compute_tile(kk[u], vv[u], base + u * WROWS, lead, cnt, lo - j0 + base + u * WROWS - lead);
        t = tn;
    }

    if (lane == 0) BUZZ_STAMP(8 + (wave & 7));
    if constexpr (!early_side<G, D>()) request_side_rows<G>(a, x, side);
    first_pass_scores<G>(a, x, prev, side);
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
    finish_split<G, D, NW>(a, x, prev, side.sc, stage, sm_m, sm_l, sm_acc, &sm_ticket);
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
        for (int g = 0; g < G; ++g) sc = add_probability(sc, logit_u[(size_t)g * a.cap + ph], M[g], iL[g]);
        a.score[ubase + ph] = sc;
    }
}

template <int G, bool NT> constexpr int unroll_for()
{
    return G == 1 ? (NT ? BUZZ_U_G1 : BUZZ_U_G1_CACHED) : (G == 2 ? BUZZ_U_G2 : (G <= 4 ? BUZZ_U_G4 : BUZZ_U_G8));
}

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
    } else {
        constexpr int RPW = 64 / (D / Elem<T>::VEC);
        // a trip covers at least 4 rows
        constexpr int US = unroll_for<G, true>() * RPW >= 4 ? unroll_for<G, true>() : 4 / RPW;     // streaming loads
        constexpr int UC = unroll_for<G, false>() * RPW >= 4 ? unroll_for<G, false>() : 4 / RPW;   // cached loads
        if (a.waves == 8) {
            if (a.streaming) BUZZ_LAUNCH((attn_split_kernel<T, D, G, US, true, 8>), grid, block, lds, st, tm, a);
            else BUZZ_LAUNCH((attn_split_kernel<T, D, G, UC, false, 8>), grid, block, lds, st, tm, a);
        } else {
            if (a.streaming) BUZZ_LAUNCH((attn_split_kernel<T, D, G, US, true, 4>), grid, block, lds, st, tm, a);
            else BUZZ_LAUNCH((attn_split_kernel<T, D, G, UC, false, 4>), grid, block, lds, st, tm, a);
        }
        return hipGetLastError();
    }
}

template <typename T, int D>
hipError_t launch_split_g(int G, const AttnArgs& a, int units, hipStream_t st, Timing tm)
{
    switch (G) {
        case 1: return launch_split_t<T, D, 1>(a, units, st, tm);
        case 2: return launch_split_t<T, D, 2>(a, units, st, tm);
        case 3: return launch_split_t<T, D, 3>(a, units, st, tm);
        case 4: return launch_split_t<T, D, 4>(a, units, st, tm);
        case 5: return launch_split_t<T, D, 5>(a, units, st, tm);
        case 6: return launch_split_t<T, D, 6>(a, units, st, tm);
        case 7: return launch_split_t<T, D, 7>(a, units, st, tm);
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
#ifdef BUZZ_TRACE
}  // namespace buzz
extern "C" int buzz_debug_trace_read(void* host, size_t bytes)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(buzz::g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
namespace buzz {
#endif
hipError_t launch_attn_split_bf16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm) { return launch_split_d<bf16_t>(D, G, a, units, st, tm); }
#else
hipError_t launch_attn_split_fp32(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm);
hipError_t launch_attn_split_fp16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm);
hipError_t launch_attn_split_bf16(int D, int G, const AttnArgs& a, int units, hipStream_t st, Timing tm);

bool attn_supported(int dtype, int D, int G)
{
    if (dtype != BUZZ_FP32 && dtype != BUZZ_FP16 && dtype != BUZZ_BF16) return false;
    if (D != 64 && D != 128 && D != 256) return false;
    return G >= 1 && G <= 8;
}

int attn_tile_rows(int dtype, int D, int G)
{
    const int vec = dtype == BUZZ_FP32 ? 4 : 8;
    const int rpw = 64 / (D / vec);
    if (G >= 2 && dtype != BUZZ_FP32) return 16;          // matrix-core kernel: 16-row tiles
    int u = G == 1 ? BUZZ_U_G1_CACHED : (G == 2 ? BUZZ_U_G2 : (G <= 4 ? BUZZ_U_G4 : BUZZ_U_G8));
    if (u * rpw < 4) u = 4 / rpw;
    return rpw * u;                                       // rows of one wave-wide trip
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
        case 3: BUZZ_LAUNCH((flush_scores_kernel<3>), grid, block, 0, st, tm, a); break;
        case 4: BUZZ_LAUNCH((flush_scores_kernel<4>), grid, block, 0, st, tm, a); break;
        case 5: BUZZ_LAUNCH((flush_scores_kernel<5>), grid, block, 0, st, tm, a); break;
        case 6: BUZZ_LAUNCH((flush_scores_kernel<6>), grid, block, 0, st, tm, a); break;
        case 7: BUZZ_LAUNCH((flush_scores_kernel<7>), grid, block, 0, st, tm, a); break;
        case 8: BUZZ_LAUNCH((flush_scores_kernel<8>), grid, block, 0, st, tm, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
#endif  // BUZZ_TU

}  // namespace buzz
