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
// see identical logits.  Plain fp32 vector arithmetic: this runs once per prompt and is not on the
// decode path.
#include "buzz_internal.h"

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

hipError_t launch_obs_scores(int dtype, int D, int /*G*/, const ObsArgs& a, int units, hipStream_t st)
{
    if (a.N <= 0 || a.t_count <= 0) return hipSuccess;
    switch (dtype) {
        case BUZZ_FP32: return launch_obs_d<BUZZ_FP32>(D, a, units, st);
        case BUZZ_FP16: return launch_obs_d<BUZZ_FP16>(D, a, units, st);
        case BUZZ_BF16: return launch_obs_d<BUZZ_BF16>(D, a, units, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace buzz
