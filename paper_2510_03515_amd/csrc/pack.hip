// Operand packing for the MFMA kernels: every contraction reads zero-padded, tile-aligned bf16
// matrices whose contraction index is contiguous, so the hot loops need no bounds checks.  These
// kernels are pure HBM copies (read once, write once).
#include "rapid_internal.h"

namespace rapid {

namespace {

struct RowLimits { int64_t R, Rpad; };

__device__ inline RowLimits row_limits(const int32_t* counts, int64_t r0, int64_t R, int64_t Rpad) {
    if (!counts) return {R, Rpad};
    int64_t m = (int64_t)counts[CNT_M] - r0, mr = (int64_t)counts[CNT_MR] - r0;
    m = m < 0 ? 0 : (m > R ? R : m);
    mr = mr < 0 ? 0 : (mr > Rpad ? Rpad : mr);
    return {m, mr};
}

// one block per destination row; 16-byte chunks (ld_dst, Cpad multiples of 8; src rows 16 B aligned
// when C % 8 == 0, otherwise the element path is taken)
__global__ void copy_pad_bf16_kernel(const bf16_t* __restrict__ src, int64_t ld_src,
                                     const int32_t* __restrict__ row_index, bf16_t* __restrict__ dst,
                                     int64_t ld_dst, int64_t R, int64_t C, int64_t Rpad, int64_t Cpad,
                                     const int32_t* __restrict__ counts, int64_t r0, int vec_ok) {
    const RowLimits lim = row_limits(counts, r0, R, Rpad);
    const int64_t r = blockIdx.x;
    if (r >= lim.Rpad) return;
    bf16_t* drow = dst + r * ld_dst;
    const bool live = r < lim.R;
    const bf16_t* srow = nullptr;
    if (live) {
        const int64_t sr = row_index ? (int64_t)row_index[r0 + r] : r;
        srow = src + sr * ld_src;
    }
    if (vec_ok) {
        const int64_t chunks = Cpad / 8, live_chunks = C / 8;
        for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (live && c < live_chunks) v = *(const uint4*)(srow + c * 8);
            *(uint4*)(drow + c * 8) = v;
        }
    } else {
        for (int64_t c = threadIdx.x; c < Cpad; c += blockDim.x)
            drow[c] = (live && c < C) ? srow[c] : (bf16_t)0;
    }
}

// 64x64 tile through LDS: dst[c][r] = src[r][c].  16-byte global accesses on both sides when the
// shapes allow (vec: ld_src, ld_dst multiples of 8, 16-byte aligned bases), elements otherwise.
// LDS rows are 66 elements (33 banks) apart: the transposed read of 8 rows x 8 columns per 64 lanes
// is conflict free.
__global__ __launch_bounds__(256) void transpose_pad_bf16_kernel(const bf16_t* __restrict__ src, int64_t ld_src,
                                                                 bf16_t* __restrict__ dst, int64_t ld_dst, int64_t R,
                                                                 int64_t C, int64_t Rpad, int64_t Cpad,
                                                                 const int32_t* __restrict__ counts, int64_t r0, int vec) {
    __shared__ bf16_t tile[64][66];
    const RowLimits lim = row_limits(counts, r0, R, Rpad);
    const int64_t rb = (int64_t)blockIdx.x * 64, cb = (int64_t)blockIdx.y * 64;
    if (rb >= lim.Rpad) return;
    if (vec) {
        for (int t = threadIdx.x; t < 512; t += 256) {          // 64 rows x 8 chunks of 8 columns
            const int rr = t >> 3, q = t & 7;
            const int64_t r = rb + rr, c = cb + q * 8;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (r < lim.R && c + 8 <= C) {
                v = *(const uint4*)(src + r * ld_src + c);
            } else if (r < lim.R && c < C) {
                bf16_t e[8];
                for (int i = 0; i < 8; ++i) e[i] = c + i < C ? src[r * ld_src + c + i] : (bf16_t)0;
                v = *(const uint4*)e;
            }
            uint32_t* p = (uint32_t*)&tile[rr][q * 8];          // 4-byte aligned: row stride 132 bytes
            p[0] = v.x; p[1] = v.y; p[2] = v.z; p[3] = v.w;
        }
        __syncthreads();
        for (int t = threadIdx.x; t < 512; t += 256) {          // 64 destination rows x 8 chunks of 8
            const int cc = t >> 3, q = t & 7;
            const int64_t c = cb + cc, r = rb + q * 8;
            if (c >= Cpad || r >= lim.Rpad) continue;
            bf16_t e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = tile[q * 8 + i][cc];
            if (r + 8 <= lim.Rpad) {
                *(uint4*)(dst + c * ld_dst + r) = *(const uint4*)e;
            } else {
                for (int i = 0; i < 8 && r + i < lim.Rpad; ++i) dst[c * ld_dst + r + i] = e[i];
            }
        }
        return;
    }
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;   // 256 threads: 64 x 4
    for (int rr = ty; rr < 64; rr += 4) {
        const int64_t r = rb + rr, c = cb + tx;
        bf16_t v = 0;
        if (r < lim.R && c < C) v = src[r * ld_src + c];
        tile[rr][tx] = v;
    }
    __syncthreads();
    for (int cc = ty; cc < 64; cc += 4) {
        const int64_t c = cb + cc, r = rb + tx;
        if (c < Cpad && r < lim.Rpad) dst[c * ld_dst + r] = tile[tx][cc];
    }
}

}  // namespace

void launch_copy_pad_bf16(const bf16_t* src, int64_t ld_src, const int32_t* row_index, bf16_t* dst,
                          int64_t ld_dst, int64_t R, int64_t C, int64_t Rpad, int64_t Cpad,
                          const int32_t* counts, int64_t r0, hipStream_t st) {
    if (Rpad <= 0) return;
    const int vec_ok = (C % 8 == 0) && (ld_src % 8 == 0) && (((uintptr_t)src) % 16 == 0);
    copy_pad_bf16_kernel<<<(unsigned)Rpad, 256, 0, st>>>(src, ld_src, row_index, dst, ld_dst, R, C, Rpad, Cpad,
                                                         counts, r0, vec_ok);
}

// Row-major [R, ld] (R multiple of RB, C multiple of 64) -> tile-blocked: block (rt, kt) holds rows
// rt*RB .. +RB, columns kt*64 .. +64 as RB contiguous 128-byte rows; blocks ordered (rt, kt).
__global__ void block_rows_bf16_kernel(const bf16_t* __restrict__ src, int64_t ld, bf16_t* __restrict__ dst, int RB,
                                       int64_t KT) {
    const int64_t rt = blockIdx.y, kt = blockIdx.x;
    const bf16_t* s = src + rt * RB * ld + kt * 64;
    bf16_t* d = dst + (rt * KT + kt) * RB * 64;
    for (int c = threadIdx.x; c < RB * 8; c += blockDim.x) {
        const int r = c >> 3, q = c & 7;
        *(uint4*)(d + r * 64 + q * 8) = *(const uint4*)(s + (int64_t)r * ld + q * 8);
    }
}
void launch_block_rows_bf16(const bf16_t* src, int64_t ld, bf16_t* dst, int64_t R, int64_t C, int RB, hipStream_t st) {
    dim3 grid((unsigned)(C / 64), (unsigned)(R / RB));
    block_rows_bf16_kernel<<<grid, 256, 0, st>>>(src, ld, dst, RB, C / 64);
}

void launch_transpose_pad_bf16(const bf16_t* src, int64_t ld_src, bf16_t* dst, int64_t ld_dst, int64_t R,
                               int64_t C, int64_t Rpad, int64_t Cpad, const int32_t* counts, int64_t r0,
                               hipStream_t st) {
    if (Rpad <= 0 || Cpad <= 0) return;
    dim3 grid((unsigned)((Rpad + 63) / 64), (unsigned)((Cpad + 63) / 64));
    const int vec = (ld_src % 8 == 0) && (ld_dst % 8 == 0) && (((uintptr_t)src) % 16 == 0) && (((uintptr_t)dst) % 16 == 0);
    transpose_pad_bf16_kernel<<<grid, 256, 0, st>>>(src, ld_src, dst, ld_dst, R, C, Rpad, Cpad, counts, r0, vec);
}

}  // namespace rapid
