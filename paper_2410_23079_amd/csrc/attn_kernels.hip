// Decode attention over the retained BUZZ cache, split over key ranges (eq. 3 / eq. 5 of the paper),
// with the append of eq. 2 fused in, followed by the combine + accumulated-score epilogue.
//
// Kernel 1 (attn_split): one block per (key-range split, unit).  A wave reads 64 x 16 B per load
// instruction = RPW consecutive cache rows, LPR = 64 / RPW lanes per row, so every load is one
// contiguous 1 KB burst.  A row's q.k dot product is an LPR-lane DPP reduction; softmax runs online
// per lane group; p.V accumulates in registers.  The scaled logit of every row goes to a scratch
// array so that the epilogue can turn it into a globally normalised probability.
// Kernel 2 (combine_score): merges the split partials into the output and adds
// sum_g softmax(...)_row to every retained row's accumulated score ("A" of Alg. 2).
#include "buzz_internal.h"

namespace buzz {
namespace {

struct bf16_t { uint16_t x; };
struct fp16_t { uint16_t x; };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;
    static __device__ inline void cvt(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};
template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ inline void cvt(const uint4& r, float* f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct Elem<fp16_t> {
    static constexpr int VEC = 8;
    static __device__ inline void cvt(const uint4& r, float* f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2_t h = __builtin_bit_cast(half2_t, w[i]);
            f[2 * i] = (float)h.x;
            f[2 * i + 1] = (float)h.y;
        }
    }
};

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

template <typename T, int D, int G, int U>
__global__ __launch_bounds__(256) void attn_split_kernel(const AttnArgs a)
{
    using E = Elem<T>;
    constexpr int VEC = E::VEC;
    constexpr int LPR = D / VEC;          // lanes per cache row
    constexpr int RPW = 64 / LPR;         // rows per wave-wide load
    constexpr int NW = 4;                 // waves per block
    constexpr int ROWB = D * (int)sizeof(T);
    constexpr int WROWS = RPW * U;        // rows one wave consumes per trip
    constexpr int TILE = NW * WROWS;
    static_assert(LPR >= 8 && LPR <= 64, "row must span 8..64 lanes");

    const int split = blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane % LPR, rs = lane / LPR;
    const int b = unit / a.Hkv, kvh = unit - b * a.Hkv;

    float qf[G][VEC];
    {
        const char* qb = (const char*)a.q + (size_t)(b * a.Hq + kvh * G) * ROWB + c * 16;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 r = *(const uint4*)(qb + (size_t)g * ROWB);
            E::cvt(r, qf[g]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) qf[g][v] *= a.scale_log2;
        }
    }

    const int j0 = split * a.rows_per_split;
    const int j1 = min(a.n, j0 + a.rows_per_split);
    const int jn = a.n - 1;
    const size_t ubase = (size_t)unit * a.cap;
    char* Kb = (char*)a.K + ubase * ROWB + c * 16;
    char* Vb = (char*)a.V + ubase * ROWB + c * 16;
    const char* knew = (const char*)a.k_new + (size_t)unit * ROWB + c * 16;
    const char* vnew = (const char*)a.v_new + (size_t)unit * ROWB + c * 16;

    float m[G], l[G], acc[G][VEC];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[g][v] = 0.f;
    }

    for (int base = j0 + wave * WROWS; base < j1; base += TILE) {
        uint4 kr[U], vr[U];
        int ph[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * RPW + rs;
            ok[u] = j < j1;
            const int jj = ok[u] ? j : j0;              // masked lanes re-read a valid row
            ph[u] = a.map.phys(jj);
            const bool is_new = jj == jn;
            const char* kp = is_new ? knew : Kb + (size_t)ph[u] * ROWB;
            const char* vp = is_new ? vnew : Vb + (size_t)ph[u] * ROWB;
            kr[u] = *(const uint4*)kp;
            vr[u] = *(const uint4*)vp;
            if (is_new && ok[u]) {                      // eq. 2: the new row joins the cache
                *(uint4*)(Kb + (size_t)a.new_phys * ROWB) = kr[u];
                *(uint4*)(Vb + (size_t)a.new_phys * ROWB) = vr[u];
                if (c == 0) a.pos[ubase + a.new_phys] = a.new_pos;
            }
        }
        float s[G][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[VEC];
            E::cvt(kr[u], kf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d = 0.f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) d = fmaf(qf[g][v], kf[v], d);
                d = row_sum<LPR>(d);
                s[g][u] = ok[u] ? d : -INFINITY;
            }
            if (ok[u] && c == 0) {
                float* lp = a.logit + (ubase + ph[u]) * G;
                if constexpr (G == 4) {
                    *(float4*)lp = make_float4(s[0][u], s[1][u], s[2][u], s[3][u]);
                } else if constexpr (G == 2) {
                    *(float2*)lp = make_float2(s[0][u], s[1][u]);
                } else if constexpr (G == 8) {
                    *(float4*)lp = make_float4(s[0][u], s[1][u], s[2][u], s[3][u]);
                    *(float4*)(lp + 4) = make_float4(s[4][u], s[5][u], s[6][u], s[7][u]);
                } else {
#pragma unroll
                    for (int g = 0; g < G; ++g) lp[g] = s[g][u];
                }
            }
        }
        float vf[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) E::cvt(vr[u], vf[u]);
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
            for (int v = 0; v < VEC; ++v) acc[g][v] *= alpha;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float p = fast_exp2(s[g][u] - mref);
                psum += p;
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[g][v] = fmaf(p, vf[u][v], acc[g][v]);
            }
            l[g] = fmaf(l[g], alpha, psum);
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
    __shared__ float sm_m[NW][G], sm_l[NW][G];
    __shared__ float sm_acc[NW][G][D];
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
    __syncthreads();
    const size_t pbase = ((size_t)unit * a.s_cap + split) * G;
    for (int i = tid; i < G * D; i += 256) {
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
        a.part_o[(pbase + g) * D + d] = o;
        if (d == 0) {
            a.part_ml[(pbase + g) * 2] = M;
            a.part_ml[(pbase + g) * 2 + 1] = L;
        }
    }
}

constexpr int kScoreRowsPerBlock = 2048;

template <int G>
__global__ __launch_bounds__(256) void combine_score_kernel(const AttnArgs a, const int D)
{
    __shared__ float sM[G], sInvL[G];
    __shared__ float sW[kMaxSplits][G];
    const int chunk = blockIdx.x, unit = blockIdx.y, tid = threadIdx.x;
    const int S = a.n_splits;
    const float* ml = a.part_ml + (size_t)unit * a.s_cap * G * 2;
    if (tid < G) {
        float M = -INFINITY;
        for (int s = 0; s < S; ++s) M = fmaxf(M, ml[(s * G + tid) * 2]);
        float L = 0.f;
        for (int s = 0; s < S; ++s) {
            const float ms = ml[(s * G + tid) * 2];
            const float w = fast_exp2(ms - M);          // M is finite: the appended row is always present
            sW[s][tid] = w;
            L = fmaf(ml[(s * G + tid) * 2 + 1], w, L);
        }
        sM[tid] = M;
        sInvL[tid] = 1.0f / L;
    }
    __syncthreads();

    const size_t ubase = (size_t)unit * a.cap;
    const int jbeg = chunk * kScoreRowsPerBlock;
    const int jend = min(a.n, jbeg + kScoreRowsPerBlock);
    for (int j = jbeg + tid; j < jend; j += 256) {
        const size_t idx = ubase + a.map.phys(j);
        float p = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) p += fast_exp2(a.logit[idx * G + g] - sM[g]) * sInvL[g];
        const float old = (j == a.n - 1) ? 0.f : a.score[idx];   // the appended row starts from zero
        a.score[idx] = old + p;
    }

    if (chunk == 0) {
        const int b = unit / a.Hkv, kvh = unit - b * a.Hkv;
        const float* po = a.part_o + (size_t)unit * a.s_cap * G * D;
        float* outp = a.out + (size_t)(b * a.Hq + kvh * G) * D;
        for (int i = tid; i < G * D; i += 256) {
            const int g = i / D, d = i - g * D;
            float o = 0.f;
            for (int s = 0; s < S; ++s) o = fmaf(sW[s][g], po[((size_t)s * G + g) * D + d], o);
            outp[(size_t)g * D + d] = o * sInvL[g];
        }
    }
}

template <int G> constexpr int unroll_for() { return G == 1 ? 8 : (G <= 4 ? 4 : 2); }

template <typename T, int D, int G>
hipError_t launch_split_t(const AttnArgs& a, int units, hipStream_t st)
{
    dim3 grid(a.n_splits, units), block(256);
    hipLaunchKernelGGL((attn_split_kernel<T, D, G, unroll_for<G>()>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_split_g(int G, const AttnArgs& a, int units, hipStream_t st)
{
    switch (G) {
        case 1: return launch_split_t<T, D, 1>(a, units, st);
        case 2: return launch_split_t<T, D, 2>(a, units, st);
        case 4: return launch_split_t<T, D, 4>(a, units, st);
        case 8: return launch_split_t<T, D, 8>(a, units, st);
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_split_d(int D, int G, const AttnArgs& a, int units, hipStream_t st)
{
    switch (D) {
        case 64: return launch_split_g<T, 64>(G, a, units, st);
        case 128: return launch_split_g<T, 128>(G, a, units, st);
        case 256: return launch_split_g<T, 256>(G, a, units, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

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
    const int u = G == 1 ? 8 : (G <= 4 ? 4 : 2);
    return 4 * rpw * u;
}

hipError_t launch_attn_split(int dtype, int D, int G, const AttnArgs& a, int units, hipStream_t st)
{
    switch (dtype) {
        case BUZZ_FP32: return launch_split_d<float>(D, G, a, units, st);
        case BUZZ_FP16: return launch_split_d<fp16_t>(D, G, a, units, st);
        case BUZZ_BF16: return launch_split_d<bf16_t>(D, G, a, units, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_combine_score(int D, int G, const AttnArgs& a, int units, hipStream_t st)
{
    dim3 grid((a.n + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock, units), block(256);
    switch (G) {
        case 1: hipLaunchKernelGGL((combine_score_kernel<1>), grid, block, 0, st, a, D); break;
        case 2: hipLaunchKernelGGL((combine_score_kernel<2>), grid, block, 0, st, a, D); break;
        case 4: hipLaunchKernelGGL((combine_score_kernel<4>), grid, block, 0, st, a, D); break;
        case 8: hipLaunchKernelGGL((combine_score_kernel<8>), grid, block, 0, st, a, D); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace buzz
