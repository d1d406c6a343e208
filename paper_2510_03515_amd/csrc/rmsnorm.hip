// Final RMSNorm folded into the operand pack of the fused call (not part of the paper's method: its
// path starts at the hidden state; the Qwen2.5 models it trains end in this norm, and the pack pass
// reads every hidden row anyway).  Forward: the packed, zero-padded bf16 operand holds
// h = x * weight / sqrt(mean(x^2) + eps) instead of a copy of x.  Backward: the dHidden kernel has
// written dL/dh (bf16) into the caller's dhidden buffer; two passes over the valid rows turn it into
// dL/dweight (fixed-order partial sums) and, in place, dL/dx.
#include "rapid_internal.h"

namespace rapid {

namespace {

constexpr int WAVE = 64;

__device__ inline float wave_sum_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// sum over the 256 threads of a block, same value in every thread, fixed order
__device__ inline float block_sum_f(float v, float* sm) {
    v = wave_sum_f(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sm[threadIdx.x / WAVE] = v;
    __syncthreads();
    return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

__device__ inline void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = __builtin_bit_cast(float, w[e] << 16);
        f[2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xffff0000u);
    }
}

// double -> float such that rounding the float to bf16 (nearest even) gives what rounding the double
// to bf16 directly would: truncate, and set the last bit if anything was cut off ("round to odd"; the
// sticky bit keeps a value just off a bf16 midpoint from landing on it)
__device__ inline float round_to_odd_f32(double v) {
    float f = (float)v;                       // nearest; repaired below if it moved the value
    if ((double)f != v && isfinite(f)) {
        uint32_t b = __builtin_bit_cast(uint32_t, f);
        const bool away = fabs((double)f) > fabs(v);   // rounded away from zero: step back to the truncation
        if (away) b -= 1u;
        b |= 1u;
        f = __builtin_bit_cast(float, b);
    }
    return f;
}

__device__ inline uint32_t pack2(float a, float b) {
    const __bf16 x = (__bf16)a, y = (__bf16)b;
    return (uint32_t)__builtin_bit_cast(unsigned short, x) | ((uint32_t)__builtin_bit_cast(unsigned short, y) << 16);
}

__device__ inline uint4 pack8(const float (&f)[8]) {
    return make_uint4(pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7]));
}

__device__ inline double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ inline double block_sum_d(double v, double* sm) {
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sm[threadIdx.x / WAVE] = v;
    __syncthreads();
    return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

// one block per destination row r < Mr (device count): rows < M hold the normalised source row
// row_index[r], the rest and the columns C .. Cpad are zero; inv_rms[r] = 1 / sqrt(mean(x^2) + eps).
// The normalised value is formed in fp64 and rounded to bf16 once: which of two neighbouring bf16
// values an element becomes is a decision, and taken from an fp32 product it would fall the other
// way than the exact value's for about one element in 40 000, each moving its row's log-prob by
// ~1e-4.  The pass is bound by its memory traffic either way.
__global__ __launch_bounds__(256) void rmsnorm_pad_bf16_kernel(const bf16_t* __restrict__ src, int64_t C,
                                                               const int32_t* __restrict__ row_index,
                                                               const bf16_t* __restrict__ weight, float eps,
                                                               bf16_t* __restrict__ dst, int64_t ld_dst, int64_t Cpad,
                                                               const int32_t* __restrict__ counts,
                                                               float* __restrict__ inv_rms, int64_t r0) {
    __shared__ double sm[4];
    const int64_t r = r0 + blockIdx.x;
    const int M = counts[CNT_M], Mr = counts[CNT_MR];
    if (r >= Mr) return;
    bf16_t* drow = dst + r * ld_dst;
    const int64_t chunks = Cpad / 8, live_chunks = C / 8;
    if (r >= M) {
        for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) *(uint4*)(drow + c * 8) = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    const bf16_t* srow = src + (int64_t)row_index[r] * C;
    double ss = 0.0;
    for (int64_t c = threadIdx.x; c < live_chunks; c += blockDim.x) {
        float x[8];
        unpack8(*(const uint4*)(srow + c * 8), x);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fma((double)x[e], (double)x[e], ss);
    }
    ss = block_sum_d(ss, sm);
    const double inv = 1.0 / sqrt(ss / (double)C + (double)eps);
    if (threadIdx.x == 0) inv_rms[r] = (float)inv;
    for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) {
        uint4 out = make_uint4(0u, 0u, 0u, 0u);
        if (c < live_chunks) {
            float x[8], g[8], h[8];
            unpack8(*(const uint4*)(srow + c * 8), x);
            unpack8(*(const uint4*)(weight + c * 8), g);
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = round_to_odd_f32((double)x[e] * inv * (double)g[e]);
            out = pack8(h);
        }
        *(uint4*)(drow + c * 8) = out;
    }
}

// dweight partials: block (rb, cb) sums dh[row][k] x[row][k] inv_rms[row] over the valid compact rows
// row0 + rb*RB .. +RB for the 8 columns of each of its threads; part[rb][k] (a block without rows writes nothing:
// `part` is zeroed beforehand)
constexpr int RB = 512;
__global__ __launch_bounds__(256) void rmsnorm_dweight_partial_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dh,
                                                                      int64_t d, const int32_t* __restrict__ row_index,
                                                                      const int32_t* __restrict__ counts,
                                                                      const float* __restrict__ inv_rms,
                                                                      float* __restrict__ part, int64_t row0) {
    const int64_t c = (int64_t)blockIdx.y * blockDim.x + threadIdx.x;   // 8-column chunk
    const int64_t r0 = row0 + (int64_t)blockIdx.x * RB;                // row blocks along x: no 65535 limit
    const int M = counts[CNT_M];
    if (c * 8 >= d || r0 >= M) return;   // the reduction reads the blocks that hold tokens only
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int64_t r1 = r0 + RB < M ? r0 + RB : M;
    for (int64_t r = r0; r < r1; ++r) {
        const int64_t pos = row_index[r];
        float xv[8], gv[8];
        unpack8(*(const uint4*)(x + pos * d + c * 8), xv);
        unpack8(*(const uint4*)(dh + pos * d + c * 8), gv);
        const float inv = inv_rms[r];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(gv[e] * inv, xv[e], acc[e]);
    }
    float* o = part + (int64_t)blockIdx.x * d + c * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = acc[e];
}

// dweight[k] = sum over all row blocks, in block order (fp64 accumulate; blocks without rows hold zeros)
__global__ void rmsnorm_dweight_reduce_kernel(const float* __restrict__ part, int64_t d, int64_t nblk,
                                              float* __restrict__ dweight) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= d) return;
    double acc = 0.0;
    for (int64_t b = 0; b < nblk; ++b) acc += (double)part[b * d + k];
    dweight[k] = (float)acc;
}

// in place, one block per valid compact row: dh -> dx = r (w dh) - x r^3 sum_k(dh_k w_k x_k) / d
__global__ __launch_bounds__(256) void rmsnorm_dx_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ dh, int64_t d,
                                                         const bf16_t* __restrict__ weight,
                                                         const int32_t* __restrict__ row_index,
                                                         const int32_t* __restrict__ counts,
                                                         const float* __restrict__ inv_rms, int64_t r0) {
    __shared__ float sm[4];
    const int64_t r = r0 + blockIdx.x;
    if (r >= counts[CNT_M]) return;
    const int64_t pos = row_index[r];
    const bf16_t* xr = x + pos * d;
    bf16_t* gr = dh + pos * d;
    const int64_t chunks = d / 8;
    float t = 0.f;
    for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) {
        float xv[8], gv[8], wv[8];
        unpack8(*(const uint4*)(xr + c * 8), xv);
        unpack8(*(const uint4*)(gr + c * 8), gv);
        unpack8(*(const uint4*)(weight + c * 8), wv);
#pragma unroll
        for (int e = 0; e < 8; ++e) t = fmaf(gv[e] * wv[e], xv[e], t);
    }
    t = block_sum_f(t, sm);   // also orders every thread's reads of the row before the writes below
    const float inv = inv_rms[r];
    const float k3 = inv * inv * inv * t / (float)d;
    for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) {
        float xv[8], gv[8], wv[8], o[8];
        unpack8(*(const uint4*)(xr + c * 8), xv);
        unpack8(*(const uint4*)(gr + c * 8), gv);
        unpack8(*(const uint4*)(weight + c * 8), wv);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = inv * wv[e] * gv[e] - xv[e] * k3;
        *(uint4*)(gr + c * 8) = pack8(o);
    }
}

}  // namespace

void launch_rmsnorm_pad_bf16(const bf16_t* src, int64_t C, const int32_t* row_index, const bf16_t* weight, float eps,
                             bf16_t* dst, int64_t ld_dst, int64_t r0, int64_t Rpad, int64_t Cpad, const int32_t* counts,
                             float* inv_rms, hipStream_t st) {
    if (Rpad <= 0) return;
    rmsnorm_pad_bf16_kernel<<<(unsigned)Rpad, 256, 0, st>>>(src, C, row_index, weight, eps, dst, ld_dst, Cpad, counts,
                                                            inv_rms, r0);
}

int64_t rmsnorm_dweight_blocks(int64_t rows_max) { return (rows_max + RB - 1) / RB; }

void launch_rmsnorm_backward(const bf16_t* x, bf16_t* dh, int64_t d, const bf16_t* weight, const int32_t* row_index,
                             const int32_t* counts, const float* inv_rms, int64_t row0, int64_t rows_max, float* part,
                             hipStream_t st) {
    if (rows_max <= 0) return;
    if (part) {
        dim3 grid((unsigned)rmsnorm_dweight_blocks(rows_max), (unsigned)((d / 8 + 255) / 256));
        rmsnorm_dweight_partial_kernel<<<grid, 256, 0, st>>>(x, dh, d, row_index, counts, inv_rms, part, row0);
    }
    rmsnorm_dx_kernel<<<(unsigned)rows_max, 256, 0, st>>>(x, dh, d, weight, row_index, counts, inv_rms, row0);
}

void launch_rmsnorm_dweight_reduce(const float* part, int64_t d, int64_t nblk, float* dweight, hipStream_t st) {
    rmsnorm_dweight_reduce_kernel<<<(unsigned)((d + 255) / 256), 256, 0, st>>>(part, d, nblk, dweight);
}

}  // namespace rapid
