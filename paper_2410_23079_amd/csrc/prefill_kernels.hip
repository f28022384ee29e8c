// Prefill scoring: the accumulated score a prompt token starts with is the sum, over the observed
// prompt queries (the last n_obs positions) and the query heads of its kv head, of the causal
// attention probability it receives (eq. 3 applied to prompt queries; the score "A" of Alg. 2).
//
// Two kernels per pass of at most kObsRows query rows (row = one query of one group member):
//   obs_row_stats : thread = query row (q kept in registers), keys streamed through LDS tiles;
//                   writes the (max, sum) of the row's logits per block of kObsKeyBlock keys;
//   obs_col_sums  : thread = key (k kept in registers), query rows streamed through LDS tiles;
//                   merges the row statistics, recomputes the logits and adds the column sums of
//                   the probabilities to the prompt scores.
// Both form a logit as an fma chain over the head dimension in the same order, so the two passes
// see identical logits.  Plain fp32 vector arithmetic; used for fp32 caches.
//
// 16-bit caches take the matrix-core pair below instead (obs_mfma_kernel<.., 1> and <.., 2>): the same two
// steps, but q.K^T runs on 16x16x32 MFMA tiles and a pass covers up to kObsPassRows queries per head, so
// scoring with every prompt query (n_obs = N) costs two launches per 4096 queries instead of two per 256
// query rows.
#include "buzz_internal.h"

#include <type_traits>

namespace buzz {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <int DT> __device__ inline void cvt16B(const uint4& r, float* f);   // 16 bytes -> 4 or 8 floats
template <> __device__ inline void cvt16B<BUZZ_FP32>(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
}
template <> __device__ inline void cvt16B<BUZZ_BF16>(const uint4& r, float* f) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
}
template <> __device__ inline void cvt16B<BUZZ_FP16>(const uint4& r, float* f) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { const half2_t h = __builtin_bit_cast(half2_t, w[i]); f[2 * i] = (float)h.x; f[2 * i + 1] = (float)h.y; }
}

// softmax scale (log2 units) of the query at prompt position `pos`; Sec. 3.5 multiplies it by log_512(pos + 1)
__device__ inline float query_scale(const ObsArgs& a, int pos)
{
    return a.log_n ? a.scale_log2 * (logf((float)(pos + 1)) * (1.0f / 6.2383246250395077f)) : a.scale_log2;
}

template <int DT> struct Vec { static constexpr int N = DT == BUZZ_FP32 ? 4 : 8; };

constexpr int kTile = 32;   // rows staged in LDS per trip

// cooperative load of `rows` rows of D elements (row r at src + row_off(r)) into fp32 LDS [kTile][D]
template <int DT, int D, typename RowPtr, typename RowScale>
__device__ inline void stage_rows(float* lds, int rows, RowScale row_scale, RowPtr row_ptr)
{
    constexpr int VEC = Vec<DT>::N, CH = D / VEC;         // 16-byte chunks per row
    for (int i = threadIdx.x; i < kTile * CH; i += 256) {
        const int r = i / CH, ch = i - r * CH;
        float f[VEC];
        float scale = 0.f;
        if (r < rows) {
            const uint4 raw = *(const uint4*)(row_ptr(r) + (size_t)ch * 16);
            cvt16B<DT>(raw, f);
            scale = row_scale(r);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) f[v] = 0.f;
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) lds[r * D + ch * VEC + v] = f[v] * scale;
    }
}

template <int D> __device__ inline float dot_lds(const float* reg, const float* lds_row)
{
    float s = 0.f;
#pragma unroll
    for (int d4 = 0; d4 < D / 4; ++d4) {
        const float4 x = *(const float4*)(lds_row + d4 * 4);
        s = fmaf(reg[d4 * 4 + 0], x.x, s);
        s = fmaf(reg[d4 * 4 + 1], x.y, s);
        s = fmaf(reg[d4 * 4 + 2], x.z, s);
        s = fmaf(reg[d4 * 4 + 3], x.w, s);
    }
    return s;
}

template <int DT, int D>
__global__ __launch_bounds__(256) void obs_row_stats_kernel(const ObsArgs a)
{
    const int G = a.Hq / a.Hkv;
    constexpr int VEC = Vec<DT>::N, ROWB = D * (DT == BUZZ_FP32 ? 4 : 2);
    __shared__ __attribute__((aligned(16))) float tile[kTile * D];
    const int kb = blockIdx.x, unit = blockIdx.y, r = threadIdx.x;
    const int b = unit / a.Hkv, kvh = unit - b * a.Hkv;
    const int R = a.t_count * G;
    const bool live = r < R;
    const int t = a.t_begin + (live ? r / G : 0), g = live ? r % G : 0;
    const int limit = a.N - a.n_obs + t;                       // last key this query may see
    const float qscale = query_scale(a, limit);
    float qreg[D];
    {
        const char* qp = (const char*)a.q_obs + ((size_t)(b * a.Hq + kvh * G + g) * a.n_obs + t) * ROWB;
#pragma unroll
        for (int ch = 0; ch < D / VEC; ++ch) {
            float f[VEC];
            cvt16B<DT>(*(const uint4*)(qp + ch * 16), f);
#pragma unroll
            for (int v = 0; v < VEC; ++v) qreg[ch * VEC + v] = f[v] * qscale;
        }
    }
    const int kbeg = kb * kObsKeyBlock, kend = min(a.N, kbeg + kObsKeyBlock);
    const char* Kb = (const char*)a.K + (size_t)unit * a.N * ROWB;
    float m = -INFINITY, l = 0.f;
    for (int k0 = kbeg; k0 < kend; k0 += kTile) {
        const int rows = min(kTile, kend - k0);
        __syncthreads();
        stage_rows<DT, D>(tile, rows, [](int) { return 1.0f; }, [&](int rr) { return Kb + (size_t)(k0 + rr) * ROWB; });
        __syncthreads();
#pragma unroll 2
        for (int kk = 0; kk < rows; ++kk) {
            if (k0 + kk > limit) break;                        // causal: later keys are invisible to this query
            const float d = dot_lds<D>(qreg, tile + kk * D);
            const float mn = fmaxf(m, d);
            l = fmaf(l, __builtin_amdgcn_exp2f(m - mn), __builtin_amdgcn_exp2f(d - mn));
            m = mn;
        }
    }
    float* st = a.stats + (((size_t)unit * gridDim.x + kb) * kObsRows + r) * 2;
    st[0] = m;
    st[1] = l;
}

template <int DT, int D>
__global__ __launch_bounds__(256) void obs_col_sums_kernel(const ObsArgs a, const int key_blocks)
{
    const int G = a.Hq / a.Hkv;
    constexpr int VEC = Vec<DT>::N, ROWB = D * (DT == BUZZ_FP32 ? 4 : 2);
    __shared__ __attribute__((aligned(16))) float tile[kTile * D];
    __shared__ float sM[kObsRows], sInvL[kObsRows];
    const int unit = blockIdx.y, tid = threadIdx.x;
    const int j = blockIdx.x * 256 + tid;                      // this thread's key
    const int b = unit / a.Hkv, kvh = unit - b * a.Hkv;
    const int R = a.t_count * G;
    {   // merge the per-key-block statistics of query row `tid`
        float M = -INFINITY;
        const float* st = a.stats + ((size_t)unit * key_blocks * kObsRows + tid) * 2;
        for (int kb = 0; kb < key_blocks; ++kb) M = fmaxf(M, st[(size_t)kb * kObsRows * 2]);
        float L = 0.f;
        for (int kb = 0; kb < key_blocks; ++kb) {
            const float mk = st[(size_t)kb * kObsRows * 2];
            L = fmaf(st[(size_t)kb * kObsRows * 2 + 1], __builtin_amdgcn_exp2f(mk - M), L);   // key 0 is always visible: M finite
        }
        sM[tid] = M;
        sInvL[tid] = 1.0f / L;
    }
    float kreg[D];
    {
        const int jj = j < a.N ? j : a.N - 1;
        const char* kp = (const char*)a.K + ((size_t)unit * a.N + jj) * ROWB;
#pragma unroll
        for (int ch = 0; ch < D / VEC; ++ch) {
            float f[VEC];
            cvt16B<DT>(*(const uint4*)(kp + ch * 16), f);
#pragma unroll
            for (int v = 0; v < VEC; ++v) kreg[ch * VEC + v] = f[v];
        }
    }
    float col = 0.f;
    for (int r0 = 0; r0 < R; r0 += kTile) {
        const int rows = min(kTile, R - r0);
        __syncthreads();
        stage_rows<DT, D>(tile, rows,
                          [&](int rr) { return query_scale(a, a.N - a.n_obs + a.t_begin + (r0 + rr) / G); },
                          [&](int rr) {
                              const int r = r0 + rr, t = a.t_begin + r / G, g = r % G;
                              return (const char*)a.q_obs + ((size_t)(b * a.Hq + kvh * G + g) * a.n_obs + t) * ROWB;
                          });
        __syncthreads();
#pragma unroll 4
        for (int rr = 0; rr < kTile; ++rr) {
            const int r = r0 + rr;
            const float d = dot_lds<D>(kreg, tile + rr * D);
            const int limit = a.N - a.n_obs + a.t_begin + r / G;
            const float p = (rr < rows && j <= limit) ? __builtin_amdgcn_exp2f(d - sM[r]) * sInvL[r] : 0.f;
            col += p;
        }
    }
    if (j < a.N) a.score[(size_t)unit * a.N + j] += col;
}


// ---------------------------------------------------------------------------------------------------
// Matrix-core prefill scoring (16-bit caches).
//
// One template serves both steps.  A wave keeps 64 "stationary" vectors in registers as the B operand of
// v_mfma_f32_16x16x32 (4 column tiles of 16) and streams tiles of 16 "moving" vectors through the A
// operand; lane (j, q) = (lane % 16, lane / 16) holds, of vector j of a tile, the 16-byte pieces 4p + q
// (a permutation of the contraction index that both operands share), and receives the four products of
// moving vectors 4q .. 4q+3 with stationary vector j.
//   step 1 (row statistics): stationary = 64 queries of one head, moving = the keys they may see;
//           every lane keeps a (reference, sum) of its query over its keys; merged over q at the end.
//   step 2 (column sums):    stationary = 64 keys, moving = the queries that may see them, head after
//           head of the group; every lane adds exp2(s - reference_i) / sum_i of its key over its queries.
// The four waves of a block take adjacent groups of 64 stationary vectors and share the moving rows: the
// block copies them, kChunk rows at a time, into one of two LDS buffers while it computes on the other
// (global loads of chunk c + 1 are issued before the tiles of chunk c and stored after them, one barrier
// per chunk).  A wave reading its tiles straight from memory, one tile ahead, spent more than half its
// time waiting for them.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes of packed 16-bit elements

template <int DT> __device__ inline f32x4 mma16(const u32x4& a, const u32x4& b, f32x4 c);
template <> __device__ inline f32x4 mma16<BUZZ_BF16>(const u32x4& a, const u32x4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
template <> __device__ inline f32x4 mma16<BUZZ_FP16>(const u32x4& a, const u32x4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

constexpr int kMmaCols = 64;            // stationary vectors per wave
constexpr int kMmaBlockCols = 256;      // ... per block of four waves

// The moving rows of one chunk in LDS.  A row occupies its D * 2 bytes plus 16: with that pitch the 16
// lanes that read the same piece of 16 different rows fall on 16 different groups of four banks.
template <int D>
struct MovingChunk {
    static constexpr int ROWB = D * 2, PIECES = ROWB / 16, PITCH = ROWB + 16;
    static constexpr int ROWS = D == 256 ? 32 : 64;                   // two buffers stay within 64 KB of LDS
    static constexpr int PER_THREAD = ROWS * PIECES / 256;            // 16-byte pieces a thread copies per chunk
    static_assert(ROWS * PIECES % 256 == 0, "the block copies whole rounds of 256 pieces");
    // issue the loads of rows row0 .. row0 + ROWS - 1 (clamped to last_row) of the array at `base`; rows are
    // contiguous, so a chunk that lies inside the array is one block of memory and piece i sits 16 i bytes
    // into it: a uniform base plus a per-thread constant, no address arithmetic per load
    static __device__ inline void request(u32x4 (&r)[PER_THREAD], const char* base, int row0, int last_row)
    {
        if (row0 + ROWS - 1 <= last_row) {
            const char* chunk = base + (size_t)row0 * ROWB;
#pragma unroll
            for (int k = 0; k < PER_THREAD; ++k) r[k] = *(const u32x4*)(chunk + (threadIdx.x + 256 * k) * 16);
        } else {
#pragma unroll
            for (int k = 0; k < PER_THREAD; ++k) {
                const int piece = threadIdx.x + 256 * k, row = piece / PIECES, col = piece - row * PIECES;
                r[k] = *(const u32x4*)(base + (size_t)min(row0 + row, last_row) * ROWB + col * 16);
            }
        }
    }
    static __device__ inline void store(char* buf, const u32x4 (&r)[PER_THREAD])
    {
#pragma unroll
        for (int k = 0; k < PER_THREAD; ++k) {
            const int piece = threadIdx.x + 256 * k, row = piece / PIECES, col = piece - row * PIECES;
            *(u32x4*)(buf + row * PITCH + col * 16) = r[k];
        }
    }
    // A operand of tile `tile` (16 rows) of the chunk for this lane
    static __device__ inline void fetch(u32x4 (&f)[D / 32], const char* buf, int tile, int j, int q)
    {
        const char* row = buf + (16 * tile + j) * PITCH + q * 16;
#pragma unroll
        for (int p = 0; p < D / 32; ++p) f[p] = *(const u32x4*)(row + p * 64);
    }
};

template <int DT, int D, int STEP, bool LOGN>
__global__ __launch_bounds__(256) void obs_mfma_kernel(const ObsArgs a)
{
    // softmax scale (log2 units) of the query at prompt position `pos`; a template flag rather than a
    // run-time one: as a run-time select the logarithm would be evaluated for every row of every tile
    auto qscale = [&](int pos) {
        return LOGN ? a.scale_log2 * (logf((float)(pos + 1)) * (1.0f / 6.2383246250395077f)) : a.scale_log2;
    };
    using MC = MovingChunk<D>;
    constexpr int ROWB = D * 2, QP = D / 32, CT = kMmaCols / 16, CH = MC::ROWS;
    constexpr bool AHEAD = D <= 128;                       // a second operand buffer fits the register budget
    __shared__ __align__(16) char sm_rows[2][CH * MC::PITCH];
    __shared__ float2 sm_stat[2][CH];                      // step 2: (reference, 1 / sum) of the chunk's queries
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform values stay in scalar registers
    const int j = lane & 15, q = lane >> 4;
    const int G = a.Hq / a.Hkv;
    const int t_end = a.t_begin + a.t_count;               // queries [t_begin, t_end) of q_obs are scored by this pass
    const int shift = a.N - a.n_obs;                       // prompt position of query t is shift + t
    auto piece = [&](const char* row, int p) { return *(const u32x4*)(row + (4 * p + q) * 16); };
    u32x4 staged[MC::PER_THREAD];

    if constexpr (STEP == 1) {
        const int head = blockIdx.x;                       // b * Hq + h
        const int b = head / a.Hq, h = head - b * a.Hq;
        const int unit = b * a.Hkv + h / G;
        // the latest queries see the most keys: their blocks go first, for all heads, so that the launch
        // ends with the short blocks (blockIdx.x, which the dispatcher advances first, is the head)
        // blockIdx.y = (group of 256 queries, part of its keys): a.key_splits blocks share a group
        const int q_blocks = (int)gridDim.y / a.key_splits;
        const int part = (int)blockIdx.y % a.key_splits;
        const int t_block = a.t_begin + (q_blocks - 1 - (int)blockIdx.y / a.key_splits) * kMmaBlockCols;
        if (t_block >= t_end) return;
        const int t_base = t_block + wave * kMmaCols;
        const bool active = t_base < t_end;                // a wave without queries still copies and synchronises
        const char* Qb = (const char*)a.q_obs + (size_t)head * a.n_obs * ROWB;
        const char* Kb = (const char*)a.K + (size_t)unit * a.N * ROWB;
        constexpr float kRefStart = -1.0e30f, kRefSlack = 1073741824.0f;   // 2^30
        u32x4 qf[CT][QP];
        int pos[CT];
        float scale[CT], m[CT], l[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const int t = t_base + 16 * ct + j;
            pos[ct] = t < t_end ? shift + t : -1;          // -1: no key is visible, the column stays empty
            scale[ct] = qscale(max(pos[ct], 0));
            const char* row = Qb + (size_t)min(t, a.n_obs - 1) * ROWB;
#pragma unroll
            for (int p = 0; p < QP; ++p) qf[ct][p] = piece(row, p);
            m[ct] = kRefStart; l[ct] = 0.f;
        }
        const int k_last = shift + min(t_base + kMmaCols, t_end) - 1;   // the wave's latest query sees keys 0 .. k_last
        const int k_free = shift + t_base;                 // keys up to here are visible to every query of the wave
        const int k_last_block = shift + min(t_block + kMmaBlockCols, t_end) - 1;
        const int n_chunks = k_last_block / CH + 1;
        const int per_part = (n_chunks + a.key_splits - 1) / a.key_splits;
        const int c_begin = part * per_part, c_end = min(n_chunks, c_begin + per_part);   // this block's chunks
        // Lazy reference: a lane sums exp2(s * scale - ref) against a reference that only moves when it has
        // to.  A chunk costs one fma, one exp2 and one add per element, straight-line code per 16 x 64 tile
        // (four independent chains of matrix instructions and the vector work on their results) with none
        // of the maximum bookkeeping, and one test at its end: if a sum of the wave has grown past kRefSlack
        // (or overflowed), the sums go back to their values before the chunk and the chunk is redone the
        // classic way, tile by tile: the reference rises to the running maximum and the sum so far is
        // rescaled.  The reference starts so low that the first chunk with a visible key always takes the
        // classic path; after it the test fails only when a logit exceeds its lane's reference by about 30
        // (log2 units).  m[] holds the reference in scaled (log2) units.
        auto products = [&](const u32x4 (&kf)[QP], int ct) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int p = 0; p < QP; ++p) acc = mma16<DT>(kf[p], qf[ct][p], acc);
            return acc;
        };
        // causal: key k0 + 4q + v against this lane's query.  An invisible key contributes 0 through a
        // select, not through a product of -inf: the log-n scale of the first prompt query is 0.
        auto tile_sum = [&](const f32x4& acc, int ct, int k0, auto masked_tag) {
            constexpr bool MASKED = decltype(masked_tag)::value;
            float e[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                e[v] = __builtin_amdgcn_exp2f(fmaf(acc[v], scale[ct], -m[ct]));
                if (MASKED && k0 + 4 * q + v > pos[ct]) e[v] = 0.f;
            }
            return (e[0] + e[1]) + (e[2] + e[3]);
        };
        auto add_tile = [&](const u32x4 (&kf)[QP], int k0, auto masked_tag) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) l[ct] += tile_sum(products(kf, ct), ct, k0, masked_tag);
        };
        auto add_tile_classic = [&](const u32x4 (&kf)[QP], int k0) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const f32x4 acc = products(kf, ct);
                float top = kRefStart;
#pragma unroll
                for (int v = 0; v < 4; ++v) top = fmaxf(top, k0 + 4 * q + v <= pos[ct] ? acc[v] * scale[ct] : kRefStart);
                // unchanged, and the factor exactly 1, where the tile brought nothing larger
                l[ct] *= __builtin_amdgcn_exp2f(fminf(m[ct] - top, 0.f));
                m[ct] = fmaxf(m[ct], top);
                l[ct] += tile_sum(acc, ct, k0, std::true_type{});
            }
        };
        MC::request(staged, Kb, c_begin * CH, a.N - 1);
        MC::store(sm_rows[c_begin & 1], staged);
        __syncthreads();
        for (int c = c_begin; c < c_end; ++c) {
            const bool more = c + 1 < c_end;
            if (more) MC::request(staged, Kb, (c + 1) * CH, a.N - 1);
            if (active) {
                float l_in[CT];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) l_in[ct] = l[ct];
                // (head_dim <= 128) the operand of tile i + 1 leaves LDS while tile i is computed; reading
                // past the wave's last tile stays inside the buffer and is never used
                u32x4 kf[2][QP];
                MC::fetch(kf[0], sm_rows[c & 1], 0, j, q);
#pragma unroll
                for (int tile = 0; tile < CH / 16; ++tile) {
                    const int k0 = c * CH + 16 * tile;
                    if (AHEAD && tile + 1 < CH / 16) MC::fetch(kf[(tile + 1) & 1], sm_rows[c & 1], tile + 1, j, q);
                    if (!AHEAD && tile > 0) MC::fetch(kf[0], sm_rows[c & 1], tile, j, q);
                    if (k0 <= k_last) {
                        // wave-uniform: does a causal boundary or the end of the query list cross this tile?
                        if (k0 + 15 > k_free || t_base + kMmaCols > t_end) add_tile(kf[AHEAD ? tile & 1 : 0], k0, std::true_type{});
                        else add_tile(kf[AHEAD ? tile & 1 : 0], k0, std::false_type{});
                    }
                }
                // the sums are nonnegative: their total passes the test only if each of them does; !(<=) also
                // catches a sum that overflowed or is not a number
                const float total = (l[0] + l[1]) + (l[2] + l[3]);
                static_assert(CT == 4, "the test adds four sums");
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(total <= kRefSlack)) != 0, 0)) {
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) l[ct] = l_in[ct];
#pragma unroll 1
                    for (int tile = 0; tile < CH / 16; ++tile) {
                        const int k0 = c * CH + 16 * tile;
                        if (k0 > k_last) break;
                        MC::fetch(kf[0], sm_rows[c & 1], tile, j, q);
                        add_tile_classic(kf[0], k0);
                    }
                }
            }
            if (more) MC::store(sm_rows[(c + 1) & 1], staged);
            __syncthreads();
        }
        if (!active) return;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {                  // merge the four key subsets of a query
#pragma unroll
            for (int off = 16; off < 64; off <<= 1) {
                const float mo = __shfl_xor(m[ct], off), lo = __shfl_xor(l[ct], off);
                const float ref = fmaxf(m[ct], mo);       // finite: every lane's reference is
                l[ct] = l[ct] * __builtin_amdgcn_exp2f(m[ct] - ref) + lo * __builtin_amdgcn_exp2f(mo - ref);
                m[ct] = ref;
            }
            const int t = t_base + 16 * ct + j;
            if (q == 0 && t < t_end) {                     // (a part without visible keys leaves (kRefStart, 0))
                float* st = a.stats + (((size_t)head * a.key_splits + part) * kObsPassRows + (t - a.t_begin)) * 2;
                st[0] = m[ct];                             // reference of the scaled logits (at most their maximum)
                st[1] = l[ct];
            }
        }
    } else {
        const int unit = blockIdx.x;                       // the earliest keys are seen by the most queries: they go first
        const int b = unit / a.Hkv, kvh = unit - b * a.Hkv;
        const int j_block = blockIdx.y * kMmaBlockCols;
        const int j_base = j_block + wave * kMmaCols;
        const bool active = j_base < a.N;
        const char* Kb = (const char*)a.K + (size_t)unit * a.N * ROWB;
        u32x4 kf[CT][QP];
        float col[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const char* row = Kb + (size_t)min(j_base + 16 * ct + j, a.N - 1) * ROWB;
#pragma unroll
            for (int p = 0; p < QP; ++p) kf[ct][p] = piece(row, p);
            col[ct] = 0.f;
        }
        // the block streams the queries from the first one that sees its first key, on the chunk grid
        // anchored at t_begin, for every head of the group in turn: item i = (head i / n_chunks, chunk i % n_chunks)
        const int t_first = max(j_block - shift, a.t_begin);
        const int t_lo = a.t_begin + (t_first - a.t_begin) / CH * CH;
        const int n_chunks = t_lo < t_end ? (t_end - t_lo + CH - 1) / CH : 0;
        const int n_items = n_chunks * G;
        const int head0 = b * a.Hq + kvh * G;
        float2 staged_stat = make_float2(0.f, 0.f);
        auto request = [&](int item) {
            const int g = item / n_chunks, t0 = t_lo + (item - g * n_chunks) * CH;
            MC::request(staged, (const char*)a.q_obs + (size_t)(head0 + g) * a.n_obs * ROWB, t0, a.n_obs - 1);
            if (threadIdx.x < CH) {                        // merge the parts: (reference, sum) -> (reference, 1 / sum)
                const float* st = a.stats + ((size_t)(head0 + g) * a.key_splits * kObsPassRows +
                                             (min(t0 + (int)threadIdx.x, t_end - 1) - a.t_begin)) * 2;
                float2 part[kObsKeySplits];
#pragma unroll
                for (int k = 0; k < kObsKeySplits; ++k)
                    part[k] = *(const float2*)(st + (size_t)min(k, a.key_splits - 1) * kObsPassRows * 2);
                float ref = part[0].x;
#pragma unroll
                for (int k = 1; k < kObsKeySplits; ++k) ref = fmaxf(ref, part[k].x);   // part 0 holds key 0: finite, l > 0
                float sum = 0.f;
#pragma unroll
                for (int k = 0; k < kObsKeySplits; ++k)
                    if (k < a.key_splits) sum = fmaf(part[k].y, __builtin_amdgcn_exp2f(part[k].x - ref), sum);
                staged_stat = make_float2(ref, 1.0f / sum);
            }
        };
        auto store = [&](int buf) {
            MC::store(sm_rows[buf], staged);
            if (threadIdx.x < CH) sm_stat[buf][threadIdx.x] = staged_stat;
        };
        auto consume_as = [&](const u32x4 (&qf)[QP], const float2 (&st)[4], int t0, auto masked_tag) {
            constexpr bool MASKED = decltype(masked_tag)::value;
            float sc[4];
            int posq[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int t = t0 + 4 * q + v;
                posq[v] = (!MASKED || t < t_end) ? shift + t : -1;
                sc[v] = qscale(max(posq[v], 0));
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int p = 0; p < QP; ++p) acc = mma16<DT>(qf[p], kf[ct][p], acc);
                const int key = j_base + 16 * ct + j;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float e = __builtin_amdgcn_exp2f(fmaf(acc[v], sc[v], -st[v].x));
                    if (MASKED && key > posq[v]) e = 0.f;
                    col[ct] = fmaf(e, st[v].y, col[ct]);
                }
            }
        };
        if (n_items > 0) {
            request(0);
            store(0);
        }
        __syncthreads();
        for (int item = 0; item < n_items; ++item) {
            const bool more = item + 1 < n_items;
            if (more) request(item + 1);
            if (active) {
                const int t_chunk = t_lo + (item % n_chunks) * CH;
                // the operand of tile i + 1 leaves LDS while tile i is computed; the statistics are read with
                // the tile itself, the products hide their latency
                u32x4 qf[2][QP];
                MC::fetch(qf[0], sm_rows[item & 1], 0, j, q);
#pragma unroll
                for (int tile = 0; tile < CH / 16; ++tile) {
                    const int t0 = t_chunk + 16 * tile;
                    if (AHEAD && tile + 1 < CH / 16) MC::fetch(qf[(tile + 1) & 1], sm_rows[item & 1], tile + 1, j, q);
                    if (!AHEAD && tile > 0) MC::fetch(qf[0], sm_rows[item & 1], tile, j, q);
                    // skipped: tiles past the last query, and tiles none of whose queries sees any key of the wave
                    if (t0 < t_end && shift + t0 + 15 >= j_base) {
                        float2 st[4];
#pragma unroll
                        for (int v = 0; v < 4; ++v) st[v] = sm_stat[item & 1][16 * tile + 4 * q + v];
                        // wave-uniform: unmasked if every query of the tile exists and sees every key of the wave
                        if (t0 + 16 > t_end || shift + t0 < j_base + kMmaCols - 1) consume_as(qf[AHEAD ? tile & 1 : 0], st, t0, std::true_type{});
                        else consume_as(qf[AHEAD ? tile & 1 : 0], st, t0, std::false_type{});
                    }
                }
            }
            if (more) store((item + 1) & 1);
            __syncthreads();
        }
        if (!active) return;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            float c = col[ct] + __shfl_xor(col[ct], 16);
            c += __shfl_xor(c, 32);
            const int key = j_base + 16 * ct + j;
            if (q == 0 && key < a.N) a.score[(size_t)unit * a.N + key] += c;
        }
    }
}

template <int DT, int D>
hipError_t launch_obs_mfma_t(const ObsArgs& a, int units, hipStream_t st, Timing tm)
{
    const int heads = units / a.Hkv * a.Hq;
    const dim3 g1(heads, (a.t_count + kMmaBlockCols - 1) / kMmaBlockCols * a.key_splits), g2(units, (a.N + kMmaBlockCols - 1) / kMmaBlockCols);
    if (a.log_n) BUZZ_LAUNCH((obs_mfma_kernel<DT, D, 1, true>), g1, dim3(256), 0, st, tm, a);
    else BUZZ_LAUNCH((obs_mfma_kernel<DT, D, 1, false>), g1, dim3(256), 0, st, tm, a);
    if (hipError_t e = hipGetLastError()) return e;
    if (a.log_n) BUZZ_LAUNCH((obs_mfma_kernel<DT, D, 2, true>), g2, dim3(256), 0, st, tm, a);
    else BUZZ_LAUNCH((obs_mfma_kernel<DT, D, 2, false>), g2, dim3(256), 0, st, tm, a);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_obs_mfma_d(int D, const ObsArgs& a, int units, hipStream_t st, Timing tm)
{
    switch (D) {
        case 64: return launch_obs_mfma_t<DT, 64>(a, units, st, tm);
        case 128: return launch_obs_mfma_t<DT, 128>(a, units, st, tm);
        case 256: return launch_obs_mfma_t<DT, 256>(a, units, st, tm);
    }
    return hipErrorInvalidValue;
}

template <int DT, int D>
hipError_t launch_obs_t(const ObsArgs& a, int units, hipStream_t st)
{
    const int key_blocks = (a.N + kObsKeyBlock - 1) / kObsKeyBlock;
    hipLaunchKernelGGL((obs_row_stats_kernel<DT, D>), dim3(key_blocks, units), dim3(256), 0, st, a);
    if (hipError_t e = hipGetLastError()) return e;
    hipLaunchKernelGGL((obs_col_sums_kernel<DT, D>), dim3((a.N + 255) / 256, units), dim3(256), 0, st, a, key_blocks);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_obs_d(int D, const ObsArgs& a, int units, hipStream_t st)
{
    switch (D) {
        case 64: return launch_obs_t<DT, 64>(a, units, st);
        case 128: return launch_obs_t<DT, 128>(a, units, st);
        case 256: return launch_obs_t<DT, 256>(a, units, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

int obs_pass_queries(int dtype, int G)
{
    return dtype == BUZZ_FP32 ? kObsRows / G : kObsPassRows;
}


hipError_t launch_obs_scores(int dtype, int D, int /*G*/, const ObsArgs& a, int units, hipStream_t st, Timing tm)
{
    if (a.N <= 0 || a.t_count <= 0) return hipSuccess;
    switch (dtype) {
        case BUZZ_FP32: return launch_obs_d<BUZZ_FP32>(D, a, units, st);
        case BUZZ_FP16: return launch_obs_mfma_d<BUZZ_FP16>(D, a, units, st, tm);
        case BUZZ_BF16: return launch_obs_mfma_d<BUZZ_BF16>(D, a, units, st, tm);
    }
    return hipErrorInvalidValue;
}

}  // namespace buzz
