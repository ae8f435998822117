// Dense pieces of the layer's backward pass (Eq. 3): the weight gradient dW = X^T S, a reduction
// over all rows of the graph, plus the two small helpers around it (activation mask on the incoming
// gradient, transpose of W for the product S W^T that the update epilogue computes).
//
// dW = X^T S is a product with a short output (d_in x d) and a contraction as long as the graph has
// rows, so it is bound by reading X and S once.  The rows are cut into contiguous spans, one per
// workgroup column; a workgroup streams its span 64 rows at a time through LDS (next stage's global
// loads are in flight while the current one is multiplied), each of its four waves owning a 16-row
// strip of the output and all its 16-column blocks in accumulators (v_mfma_f32_16x16x4_f32: lane
// (i = l%16, q = l/16) supplies A(i, k=q) = X[row q][i] and B(k=q, i) = S[row q][i]).  Every span
// writes its partial product and a second kernel adds the partials in span order, so the result
// does not depend on scheduling.
#include "common.hpp"

namespace hcspmm {

typedef float v4f_bw __attribute__((ext_vector_type(4)));

constexpr int kTnRows = 64;       // rows of X and S per stage
constexpr int kTnM = 64;          // output rows (columns of X) per workgroup: 16 per wave
constexpr int kTnLdx = kTnM + 16; // LDS row pitches: = 16 mod 64, so the four k rows of an operand read fall in distinct banks

template <int NB> struct TnShape {
    static constexpr int N = NB * 16;                               // output columns (columns of S) per workgroup
    static constexpr int LDS_S = (N + 63) / 64 * 64 + 16;
    static constexpr int XV = kTnRows * kTnM / 4 / 256;             // float4 per thread per stage, X
    static constexpr int SV = (kTnRows * N / 4 + 255) / 256;        // float4 per thread per stage, S
};

// one float4 of a row-major matrix with zero fill outside [0, rows) x [0, cols); vec: rows are 16-byte aligned
__device__ inline float4 load4_guarded(const float* __restrict__ p, int64_t ld, int64_t r, int64_t rows, int c, int cols,
                                       bool vec)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r >= rows || c >= cols) return v;
    const float* __restrict__ q = p + r * ld + c;
    if (vec && c + 4 <= cols) return *reinterpret_cast<const float4*>(q);
    v.x = q[0];
    if (c + 1 < cols) v.y = q[1];
    if (c + 2 < cols) v.z = q[2];
    if (c + 3 < cols) v.w = q[3];
    return v;
}

template <int NB>
__global__ __launch_bounds__(256) void k_gemm_tn(int64_t n_rows, int64_t rows_per_span, const float* __restrict__ X,
                                                 int64_t ldx, int32_t d_in, const float* __restrict__ S, int64_t lds_,
                                                 int32_t d, float* __restrict__ partial, int xvec, int svec)
{
    using T = TnShape<NB>;
    extern __shared__ float smem[];
    float* __restrict__ xs = smem;                                  // kTnRows x kTnLdx
    float* __restrict__ ss = smem + kTnRows * kTnLdx;               // kTnRows x LDS_S
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i = lane & 15, q = lane >> 4;
    const int m0 = blockIdx.y * kTnM, n0 = blockIdx.z * 256;
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_span;
    const int64_t r_end = min(n_rows, r_begin + rows_per_span);
    v4f_bw acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = (v4f_bw){0.f, 0.f, 0.f, 0.f};
    float4 xr[T::XV], sr[T::SV];
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int j = 0; j < T::XV; ++j) {
            const int idx = tid + 256 * j, r = idx / (kTnM / 4), c = (idx % (kTnM / 4)) * 4;
            xr[j] = load4_guarded(X, ldx, r0 + r, r_end, m0 + c, d_in, xvec);
        }
#pragma unroll
        for (int j = 0; j < T::SV; ++j) {
            const int idx = tid + 256 * j, r = idx / (T::N / 4), c = (idx % (T::N / 4)) * 4;
            sr[j] = r < kTnRows ? load4_guarded(S, lds_, r0 + r, r_end, n0 + c, d, svec) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    if (r_begin < r_end) fetch(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kTnRows) {
        __syncthreads();                                            // the previous stage's reads are done
#pragma unroll
        for (int j = 0; j < T::XV; ++j) {
            const int idx = tid + 256 * j, r = idx / (kTnM / 4), c = (idx % (kTnM / 4)) * 4;
            *reinterpret_cast<float4*>(&xs[r * kTnLdx + c]) = xr[j];
        }
#pragma unroll
        for (int j = 0; j < T::SV; ++j) {
            const int idx = tid + 256 * j, r = idx / (T::N / 4), c = (idx % (T::N / 4)) * 4;
            if (r < kTnRows) *reinterpret_cast<float4*>(&ss[r * T::LDS_S + c]) = sr[j];
        }
        __syncthreads();
        if (r0 + kTnRows < r_end) fetch(r0 + kTnRows);
#pragma unroll 4
        for (int k = 0; k < kTnRows; k += 4) {
            const float a = xs[(k + q) * kTnLdx + 16 * wave + i];
#pragma unroll
            for (int b = 0; b < NB; ++b)
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, ss[(k + q) * T::LDS_S + 16 * b + i], acc[b], 0, 0, 0);
        }
    }
    // partial[span][m][n], m < d_in, n < d; accumulator r of lane (i, q) is output (16*wave + 4q + r, 16b + i)
    float* __restrict__ out = partial + (int64_t)blockIdx.x * d_in * d;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int n = n0 + 16 * b + i;
        if (n >= d) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + 16 * wave + 4 * q + r;
            if (m < d_in) out[(int64_t)m * d + n] = acc[b][r];
        }
    }
}

// out[e] = sum over spans of partial[span][e], in an order that depends only on the span count: 16
// threads per output each add every 16th span in ascending order, then one of them adds the 16 sums
// in ascending order.
__global__ __launch_bounds__(256) void k_sum_partials(int32_t n_spans, int64_t count, int32_t d,
                                                      const float* __restrict__ partial, float* __restrict__ out,
                                                      int64_t ldo)
{
    __shared__ float red[16][17];
    const int o = threadIdx.x & 15, j = threadIdx.x >> 4;
    const int64_t e = (int64_t)blockIdx.x * 16 + o;
    float s = 0.f;
    if (e < count) {
#pragma unroll 4
        for (int32_t p = j; p < n_spans; p += 16) s += partial[(int64_t)p * count + e];
    }
    red[j][o] = s;
    __syncthreads();
    if (j == 0 && e < count) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 16; ++k) t += red[k][o];
        out[(e / d) * ldo + e % d] = t;
    }
}

int32_t gemm_tn_spans(int64_t n_rows, int32_t d_in, int32_t d)
{
    const int64_t gy = (d_in + kTnM - 1) / kTnM, gz = (d + 255) / 256;
    const int64_t stages = (n_rows + kTnRows - 1) / kTnRows;
    int64_t spans = 1024 / (gy * gz);                                // about four workgroups per CU in all
    if (spans > stages / 8) spans = stages / 8;                      // at least eight stages per span
    if (spans < 1) spans = 1;
    return (int32_t)spans;
}

// dW (d_in x d, pitch lddw) = X^T S for X n_rows x d_in and S n_rows x d; partial holds
// gemm_tn_spans(n_rows, d_in, d) * d_in * d floats.
hipError_t launch_gemm_tn(int64_t n_rows, const float* X, int64_t ldx, int32_t d_in, const float* S, int64_t lds_,
                          int32_t d, float* dW, int64_t lddw, float* partial, hipStream_t s)
{
    const int32_t spans = gemm_tn_spans(n_rows, d_in, d);
    const int64_t stages = (n_rows + kTnRows - 1) / kTnRows;
    const int64_t rows_per_span = (stages + spans - 1) / spans * kTnRows;
    const dim3 grid((unsigned)spans, (unsigned)((d_in + kTnM - 1) / kTnM), (unsigned)((d + 255) / 256));
    const int xvec = ldx % 4 == 0 && (uintptr_t)X % 16 == 0, svec = lds_ % 4 == 0 && (uintptr_t)S % 16 == 0;
    const int blocks16 = (min(d, 256) + 15) / 16;
#define HC_TN(NB)                                                                                              \
    {                                                                                                          \
        const size_t lds_bytes = (size_t)(kTnRows * kTnLdx + kTnRows * TnShape<NB>::LDS_S) * sizeof(float);    \
        static bool attr_set = false;      /* once per process: later calls may run under stream capture */    \
        if (!attr_set) {                                                                                       \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_tn<NB>),                  \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);    \
            if (e != hipSuccess) return e;                                                                     \
            attr_set = true;                                                                                   \
        }                                                                                                      \
        hipLaunchKernelGGL((k_gemm_tn<NB>), grid, dim3(256), lds_bytes, s, n_rows, rows_per_span, X, ldx, d_in, S, lds_, \
                           d, partial, xvec, svec);                                                            \
    }
    if (blocks16 <= 1) HC_TN(1)
    else if (blocks16 <= 2) HC_TN(2)
    else if (blocks16 <= 4) HC_TN(4)
    else if (blocks16 <= 8) HC_TN(8)
    else HC_TN(16)
#undef HC_TN
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t count = (int64_t)d_in * d;
    hipLaunchKernelGGL(k_sum_partials, dim3((unsigned)((count + 15) / 16)), dim3(256), 0, s, spans, count, d, partial,
                       dW, lddw);
    return hipGetLastError();
}

// Gm = G where the forward output is positive, else 0 (derivative of max(0, .)); Gm is n x d, pitch ldo (it may be G
// itself).  VEC = 4: d and all pitches are multiples of 4 and the bases 16-byte aligned.
template <int VEC>
__global__ __launch_bounds__(256) void k_relu_mask(int64_t n, int32_t d, const float* G, int64_t ldg,
                                                   const float* __restrict__ Yf, int64_t ldy, float* Gm, int64_t ldo)
{
    const int per_row = d / VEC;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n * per_row) return;
    const int64_t r = e / per_row;
    const int c = (int)(e % per_row) * VEC;
    if constexpr (VEC == 4) {
        const float4 g = *reinterpret_cast<const float4*>(G + r * ldg + c);
        const float4 y = *reinterpret_cast<const float4*>(Yf + r * ldy + c);
        *reinterpret_cast<float4*>(Gm + r * ldo + c) =
            make_float4(y.x > 0.f ? g.x : 0.f, y.y > 0.f ? g.y : 0.f, y.z > 0.f ? g.z : 0.f, y.w > 0.f ? g.w : 0.f);
    } else {
        Gm[r * ldo + c] = Yf[r * ldy + c] > 0.f ? G[r * ldg + c] : 0.f;
    }
}

hipError_t launch_relu_mask(int64_t n, int32_t d, const float* G, int64_t ldg, const float* Yf, int64_t ldy, float* Gm,
                            int64_t ldo, hipStream_t s)
{
    if (n <= 0 || d <= 0) return hipSuccess;
    const bool vec = d % 4 == 0 && ldg % 4 == 0 && ldy % 4 == 0 && ldo % 4 == 0 && (uintptr_t)G % 16 == 0 &&
                     (uintptr_t)Yf % 16 == 0 && (uintptr_t)Gm % 16 == 0;
    const int64_t count = n * (vec ? d / 4 : d);
    const dim3 grid((unsigned)((count + 255) / 256));
    if (vec) hipLaunchKernelGGL(k_relu_mask<4>, grid, dim3(256), 0, s, n, d, G, ldg, Yf, ldy, Gm, ldo);
    else hipLaunchKernelGGL(k_relu_mask<1>, grid, dim3(256), 0, s, n, d, G, ldg, Yf, ldy, Gm, ldo);
    return hipGetLastError();
}

// Wt (cols x rows, pitch rows) = transpose of W (rows x cols, pitch ldw); W is small
__global__ __launch_bounds__(256) void k_transpose(int32_t rows, int32_t cols, const float* __restrict__ W, int64_t ldw,
                                                   float* __restrict__ Wt)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)rows * cols) return;
    const int64_t c = e / rows, r = e % rows;
    Wt[e] = W[r * ldw + c];
}

hipError_t launch_transpose(int32_t rows, int32_t cols, const float* W, int64_t ldw, float* Wt, hipStream_t s)
{
    const int64_t count = (int64_t)rows * cols;
    hipLaunchKernelGGL(k_transpose, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, rows, cols, W, ldw, Wt);
    return hipGetLastError();
}

}  // namespace hcspmm
