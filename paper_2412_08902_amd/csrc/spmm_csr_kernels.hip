// Scalar path: SpMM straight from CSR for the windows the selector leaves on the vector ALUs
// (Alg. 1 gives the arithmetic, Alg. 3 the mapping idea: a group of lanes owns one output row and
// each lane one slice of the dense width, so X rows are read as whole contiguous segments).
//
// wave64 mapping: a group of LPR lanes owns a row, every lane holds VEC consecutive output
// columns, so a 64-lane wave works on 64/LPR rows (short rows) or on 64/LPR non-zeros of the same
// row (long rows) per load instruction.  Column indices and values are fetched LPR at a time with
// one coalesced load per group and handed round with cross-lane reads; X itself is read directly
// from global memory / L2 (the paper found staging X in shared memory a loss on this path).
#include "common.hpp"

namespace hcspmm {

template <int VEC> struct VecT;
template <> struct VecT<4> { using type = float4; };
template <> struct VecT<2> { using type = float2; };
template <> struct VecT<1> { using type = float; };

template <int VEC> __device__ inline void vzero(float (&a)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) a[i] = 0.f;
}

template <int VEC> __device__ inline void vload(const float* __restrict__ p, float (&x)[VEC])
{
    using V = typename VecT<VEC>::type;
    V v = *reinterpret_cast<const V*>(p);
    const float* f = reinterpret_cast<const float*>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) x[i] = f[i];
}

template <int VEC> __device__ inline void vstore(float* __restrict__ p, const float (&x)[VEC], int relu)
{
    using V = typename VecT<VEC>::type;
    V v;
    float* f = reinterpret_cast<float*>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) f[i] = relu ? fmaxf(x[i], 0.f) : x[i];
    *reinterpret_cast<V*>(p) = v;
}

// Accumulate  acc += sum_{k in [kb, ke) taken LPR at a time with stride `stride`} val[k] * X[col[k], c .. c+VEC)
// for the group's lane `lig`.  All lanes of a group execute this together.
template <int LPR, int VEC>
__device__ inline void row_accumulate(int kb, int ke, int stride, int lig, bool col_ok,
                                      const int32_t* __restrict__ colind, const float* __restrict__ vals,
                                      const float* __restrict__ Xc /* X + column offset of this lane */, int64_t ldx,
                                      float (&acc)[VEC])
{
    constexpr int U = LPR < 8 ? LPR : 8;
    for (int k0 = kb; k0 < ke; k0 += stride) {
        const int k = k0 + lig;
        const int32_t mc = k < ke ? colind[k] : 0;
        const float mv = k < ke ? vals[k] : 0.f;
        const int cnt = min(LPR, ke - k0);
        int t0 = 0;
        for (; t0 + U <= cnt; t0 += U) {
            float x[U][VEC];
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t c = __shfl(mc, t0 + u, LPR);
                v[u] = __shfl(mv, t0 + u, LPR);
                if (col_ok) vload<VEC>(Xc + (int64_t)c * ldx, x[u]);
                else vzero<VEC>(x[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = fmaf(v[u], x[u][i], acc[i]);
        }
        for (; t0 < cnt; ++t0) {
            const int32_t c = __shfl(mc, t0, LPR);
            const float v = __shfl(mv, t0, LPR);
            float x[VEC];
            if (col_ok) vload<VEC>(Xc + (int64_t)c * ldx, x);
            else vzero<VEC>(x);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaf(v, x[i], acc[i]);
        }
    }
}

// ---- short rows: one group of LPR lanes per row -------------------------------------------------
template <int LPR, int VEC>
__global__ __launch_bounds__(256) void k_csr_short(int32_t n_items, const int32_t* __restrict__ row_list,
                                                   const uint8_t* __restrict__ route, SpmmArgs a)
{
    constexpr int GPB = 256 / LPR;
    const int64_t item = (int64_t)blockIdx.x * GPB + threadIdx.x / LPR;
    const int lig = threadIdx.x % LPR;
    if (item >= n_items) return;
    const int32_t row = row_list ? row_list[item] : (int32_t)item;
    const int32_t s = a.rowptr[row], e = a.rowptr[row + 1];
    if (!row_list && (route[row / kH] != 0 || e - s > kLongRow)) return;
    const float* __restrict__ X = static_cast<const float*>(a.X);
    for (int c0 = 0; c0 < a.d; c0 += LPR * VEC) {
        const int c = c0 + lig * VEC;
        const bool col_ok = c < a.d;
        float acc[VEC];
        vzero<VEC>(acc);
        row_accumulate<LPR, VEC>(s, e, LPR, lig, col_ok, a.colind, a.vals, X + c, a.ldx, acc);
        if (col_ok) vstore<VEC>(a.Y + (int64_t)row * a.ldy + c, acc, a.relu);
    }
}

// ---- long rows: one workgroup per segment of a row ----------------------------------------------
template <int LPR, int VEC>
__global__ __launch_bounds__(256) void k_csr_long(const Segment* __restrict__ segs, float* __restrict__ partial,
                                                  SpmmArgs a)
{
    constexpr int G = 256 / LPR;
    __shared__ float red[256 * VEC];
    const Segment sg = segs[blockIdx.x];
    const int g = threadIdx.x / LPR, lig = threadIdx.x % LPR;
    const float* __restrict__ X = static_cast<const float*>(a.X);
    for (int c0 = 0; c0 < a.d; c0 += LPR * VEC) {
        const int c = c0 + lig * VEC;
        const bool col_ok = c < a.d;
        float acc[VEC];
        vzero<VEC>(acc);
        row_accumulate<LPR, VEC>(sg.k_begin + g * LPR, sg.k_end, G * LPR, lig, col_ok, a.colind, a.vals, X + c,
                                 a.ldx, acc);
        // fixed-order tree over the G groups: the result does not depend on scheduling
#pragma unroll
        for (int i = 0; i < VEC; ++i) red[(g * LPR + lig) * VEC + i] = acc[i];
        __syncthreads();
        for (int st = G / 2; st > 0; st >>= 1) {
            if (g < st) {
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    red[(g * LPR + lig) * VEC + i] += red[((g + st) * LPR + lig) * VEC + i];
            }
            __syncthreads();
        }
        if (g == 0 && col_ok) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = red[lig * VEC + i];
            if (sg.slot < 0) vstore<VEC>(a.Y + (int64_t)sg.row * a.ldy + c, acc, a.relu);
            else vstore<VEC>(partial + (int64_t)sg.slot * a.d + c, acc, 0);
        }
        __syncthreads();
    }
}

// ---- rows cut into several segments: add the partial rows in segment order ----------------------
__global__ __launch_bounds__(256) void k_reduce_partials(int32_t n_multi, const MultiRow* __restrict__ multi,
                                                         const float* __restrict__ partial, SpmmArgs a)
{
    const MultiRow m = multi[blockIdx.x];
    for (int c = threadIdx.x; c < a.d; c += 256) {
        float acc = 0.f;
        for (int q = 0; q < m.n_slots; ++q) acc += partial[(int64_t)(m.first_slot + q) * a.d + c];
        a.Y[(int64_t)m.row * a.ldy + c] = a.relu ? fmaxf(acc, 0.f) : acc;
    }
}

// ---- dispatch -------------------------------------------------------------------------------------
struct CsrShape { int lpr, vec; };

static CsrShape pick_shape(const SpmmArgs& a, const float* partial)
{
    int vec = 1;
    const uintptr_t px = (uintptr_t)a.X, py = (uintptr_t)a.Y, pp = (uintptr_t)partial;
    if (a.d % 4 == 0 && a.ldx % 4 == 0 && a.ldy % 4 == 0 && px % 16 == 0 && py % 16 == 0 && pp % 16 == 0) vec = 4;
    else if (a.d % 2 == 0 && a.ldx % 2 == 0 && a.ldy % 2 == 0 && px % 8 == 0 && py % 8 == 0 && pp % 8 == 0) vec = 2;
    const int lanes = (a.d + vec - 1) / vec;       // lanes needed to cover the width once
    int lpr = 4;
    while (lpr < 64 && lpr < lanes) lpr <<= 1;
    return {lpr, vec};
}

#define HC_CSR_DISPATCH(FN)                                                                        \
    switch (sh.vec * 100 + sh.lpr) {                                                               \
        case 404: FN(4, 4); break;                                                                 \
        case 408: FN(8, 4); break;                                                                 \
        case 416: FN(16, 4); break;                                                                \
        case 432: FN(32, 4); break;                                                                \
        case 464: FN(64, 4); break;                                                                \
        case 204: FN(4, 2); break;                                                                 \
        case 208: FN(8, 2); break;                                                                 \
        case 216: FN(16, 2); break;                                                                \
        case 232: FN(32, 2); break;                                                                \
        case 264: FN(64, 2); break;                                                                \
        case 104: FN(4, 1); break;                                                                 \
        case 108: FN(8, 1); break;                                                                 \
        case 116: FN(16, 1); break;                                                                \
        case 132: FN(32, 1); break;                                                                \
        default: FN(64, 1); break;                                                                 \
    }

hipError_t launch_csr_short(const SpmmArgs& a, int32_t n_items, const int32_t* row_list, const uint8_t* route,
                            hipStream_t s)
{
    if (n_items <= 0) return hipSuccess;
    const CsrShape sh = pick_shape(a, nullptr);
#define HC_LAUNCH_SHORT(L, V)                                                                      \
    hipLaunchKernelGGL((k_csr_short<L, V>), dim3((unsigned)(((int64_t)n_items + (256 / L) - 1) / (256 / L))),     \
                       dim3(256), 0, s, n_items, row_list, route, a)
    HC_CSR_DISPATCH(HC_LAUNCH_SHORT)
#undef HC_LAUNCH_SHORT
    return hipGetLastError();
}

hipError_t launch_csr_long(const SpmmArgs& a, int32_t n_segs, const Segment* segs, float* partial, hipStream_t s)
{
    if (n_segs <= 0) return hipSuccess;
    const CsrShape sh = pick_shape(a, partial);
#define HC_LAUNCH_LONG(L, V) hipLaunchKernelGGL((k_csr_long<L, V>), dim3(n_segs), dim3(256), 0, s, segs, partial, a)
    HC_CSR_DISPATCH(HC_LAUNCH_LONG)
#undef HC_LAUNCH_LONG
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const SpmmArgs& a, int32_t n_multi, const MultiRow* multi, const float* partial,
                                  hipStream_t s)
{
    if (n_multi <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_reduce_partials, dim3(n_multi), dim3(256), 0, s, n_multi, multi, partial, a);
    return hipGetLastError();
}

}  // namespace hcspmm
