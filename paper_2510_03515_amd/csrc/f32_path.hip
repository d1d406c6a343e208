// fp32 path: the same pipeline for float inputs, built from one strided LDS-tiled contraction that
// accumulates in fp64 plus two row-wise kernels over a materialised row chunk of logits.  It is the
// accuracy path (small shapes, tolerance 1e-5), not the throughput path.
#include "rapid_internal.h"

namespace rapid {

namespace {

constexpr int TS = 16;

__global__ void f32_gemm_kernel(F32Gemm g) {
    __shared__ float As[TS][TS + 1];
    __shared__ float Bs[TS][TS + 1];
    int64_t I = g.I, Kd = g.Kd;
    if (g.counts) {
        int64_t lim = (int64_t)g.counts[CNT_M] - g.i0;
        lim = lim < 0 ? 0 : lim;
        if (g.limit_k) Kd = lim < Kd ? lim : Kd;
        else I = lim < I ? lim : I;
    }
    const int64_t ib = (int64_t)blockIdx.y * TS, jb = (int64_t)blockIdx.x * TS;
    if (ib >= I) return;
    if (g.limit_k && Kd == 0 && g.beta) return;
    const int ty = threadIdx.y, tx = threadIdx.x;
    const int64_t i = ib + ty, j = jb + tx;
    double acc = 0.0;
    for (int64_t k0 = 0; k0 < Kd; k0 += TS) {
        // A tile: element (i = ib + ty, k = k0 + tx)
        {
            const int64_t ai = ib + ty, ak = k0 + tx;
            float v = 0.f;
            if (ai < I && ak < Kd) {
                const int64_t r = g.a_imap ? (int64_t)g.a_imap[g.i0 + ai] : ai;
                const int64_t kk = g.a_kmap ? (int64_t)g.a_kmap[g.i0 + ak] : ak;
                v = g.A[r * g.sa_i + kk * g.sa_k];
            }
            As[ty][tx] = v;
        }
        {
            const int64_t bk = k0 + ty, bj = jb + tx;
            float v = 0.f;
            if (bk < Kd && bj < g.J) v = g.B[bk * g.sb_k + bj * g.sb_j];
            Bs[ty][tx] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TS; ++kk) acc += (double)As[ty][kk] * (double)Bs[kk][tx];
        __syncthreads();
    }
    if (i < I && j < g.J) {
        const int64_t r = g.c_rows ? (int64_t)g.c_rows[g.i0 + i] : i;
        float* p = g.C + r * g.sc_i + j * g.sc_j;
        const double v = acc * (double)g.alpha;
        *p = (float)(g.beta ? (double)*p + v : v);
    }
}

__device__ inline double block_reduce(double v, double* sm, bool is_max) {
    for (int o = 32; o > 0; o >>= 1) {
        const double u = __shfl_xor(v, o, 64);
        v = is_max ? fmax(v, u) : v + u;
    }
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[w] = v;
    __syncthreads();
    double r = sm[0];
    for (int q = 1; q < nw; ++q) r = is_max ? fmax(r, sm[q]) : r + sm[q];
    return r;
}

// one block per chunk row: lse over the V logits, log-prob of the sampled token
__global__ void f32_row_lse_kernel(const float* __restrict__ z, int64_t V, int64_t m0,
                                   const int32_t* __restrict__ tokc, const int32_t* __restrict__ row_index,
                                   const int32_t* __restrict__ counts, float* __restrict__ lse_c,
                                   float* __restrict__ logp_out, float* __restrict__ lse_out) {
    __shared__ double sm[16];
    const int64_t jl = blockIdx.x, j = m0 + jl;
    if (j >= counts[CNT_M]) return;
    const float* row = z + jl * V;
    double mx = -INFINITY;
    for (int64_t v = threadIdx.x; v < V; v += blockDim.x) mx = fmax(mx, (double)row[v]);
    mx = block_reduce(mx, sm, true);
    double sum = 0.0;
    for (int64_t v = threadIdx.x; v < V; v += blockDim.x) sum += exp((double)row[v] - mx);
    sum = block_reduce(sum, sm, false);
    if (threadIdx.x == 0) {
        const double lse = mx + log(sum);
        lse_c[j] = (float)lse;
        const int32_t pos = row_index[j];
        logp_out[pos] = (float)((double)row[tokc[j]] - lse);
        if (lse_out) lse_out[pos] = (float)lse;
    }
}

__global__ void f32_dz_kernel(float* __restrict__ z, int64_t V, int64_t m0, const int32_t* __restrict__ tokc,
                              const float* __restrict__ lse_c, const float* __restrict__ rowg, float inv_temp,
                              const int32_t* __restrict__ counts) {
    const int64_t jl = blockIdx.x, j = m0 + jl;
    if (j >= counts[CNT_M]) return;
    float* row = z + jl * V;
    const double lse = (double)lse_c[j];
    const double gj = (double)rowg[j] * (double)inv_temp;
    const int tok = tokc[j];
    for (int64_t v = threadIdx.x; v < V; v += blockDim.x) {
        const double p = exp((double)row[v] - lse);
        row[v] = (float)(gj * ((v == tok ? 1.0 : 0.0) - p));
    }
}

}  // namespace

void launch_f32_gemm(const F32Gemm& g, hipStream_t st) {
    if (g.I <= 0 || g.J <= 0) return;
    dim3 grid((unsigned)((g.J + TS - 1) / TS), (unsigned)((g.I + TS - 1) / TS));
    f32_gemm_kernel<<<grid, dim3(TS, TS), 0, st>>>(g);
}

void launch_f32_row_lse(const float* z, int64_t V, int64_t rows, int64_t m0, const int32_t* tokc,
                        const int32_t* row_index, const int32_t* counts, float* lse_c, float* logp_out,
                        float* lse_out, hipStream_t st) {
    if (rows > 0)
        f32_row_lse_kernel<<<(unsigned)rows, 256, 0, st>>>(z, V, m0, tokc, row_index, counts, lse_c, logp_out,
                                                           lse_out);
}

void launch_f32_dz(float* z, int64_t V, int64_t rows, int64_t m0, const int32_t* tokc, const float* lse_c,
                   const float* rowg, float inv_temp, const int32_t* counts, hipStream_t st) {
    if (rows > 0) f32_dz_kernel<<<(unsigned)rows, 256, 0, st>>>(z, V, m0, tokc, lse_c, rowg, inv_temp, counts);
}

}  // namespace rapid
