// bf16 MFMA contractions of the hot path for gfx950 (CDNA4): one persistent, software-pipelined
// main loop and four epilogues.
//   fwd_lse : logits tile  -> per-slot (max, sum exp) of the streaming log-softmax + gathered logit
//   dz      : logits tile  -> dz = g (onehot - softmax) / temperature, written as bf16
//   dh      : dH = dz . W^T          (contraction over the vocabulary)
//   dw      : dW (+)= H^T . dz       (contraction over the tokens of a row chunk)
//
// Tiling.  C[i][j] = sum_k A(i,k) B(j,k).  A workgroup of four 64-lane waves (2 x 2) owns a
// (64 WI) x (64 WJ) tile, each wave WI x WJ blocks of 32 x 32 computed with
// v_mfma_f32_32x32x16_bf16; the 256 x 256 tile fills the register file (256 accumulator registers
// per lane) and is the largest tile a CU can hold, which minimises L2 -> LDS bytes per flop.
// K advances 64 elements per step through two LDS stages of 64 KiB (one barrier per step); tiles
// arrive by global_load_lds_dwordx4 (memory -> LDS without passing through registers).
//
// Persistence.  The grid is one workgroup per CU.  Workgroup w runs on XCD w % 8 (hardware deals
// workgroup ids round-robin to the 8 XCDs, each with its own 4 MiB L2) and walks the tiles
// xcd * per + slot, + 32, + 64 ... of that XCD's contiguous share of a grouped tile order, so the
// 32 workgroups resident on an XCD always work on 32 neighbouring tiles and share operand panels
// out of L2.  The first K step of the next tile is requested while the last step of the current
// tile is computed, so the epilogue overlaps the memory latency of the next tile.
//
// LDS layouts (both conflict-free for a 256-byte LDS cycle, checked with SQ_LDS_BANK_CONFLICT):
//  * row-major operands ([row][k], k contiguous): a tile row of a step is 128 bytes = 8 chunks of
//    16 bytes; chunk c of row r sits at position c ^ ((r >> 1) & 7); fragments are read with
//    ds_read_b128 (8 consecutive k of one row per lane).
//  * k-major operands ([k][column], used by dW where the contraction index is the token row): a
//    step is 64 rows of 2 COLS bytes, cut into 64-byte segments with segment g of row r at
//    position g ^ (r % SEGS); fragments are read with ds_read_b64_tr_b16, the LDS transpose read:
//    in each group of 16 lanes, lane l receives element (l % 4) of the 8-byte pieces addressed by
//    lanes l/4, l/4 + 4, l/4 + 8, l/4 + 12.  Pointing lane s at row s / 4, columns 4 (s % 4) .. + 3
//    hands lane l column l and 4 consecutive rows: the per-lane slice of an MFMA operand.
//
// Accumulator layout of a 32 x 32 block (lane l, register v): j = l % 32,
// i = 8 (v / 4) + 4 (l / 32) + v % 4: a lane owns runs of 4 consecutive i for one j, so every
// epilogue keeps j = the token row (per-lane scalars: lse, coefficient, token id, output row).
#include "rapid_internal.h"

namespace rapid {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int NT = 256;              // threads per workgroup
constexpr float LOG2E = 1.4426950408889634f;

template <int WI, int WJ>
struct Shape {
    static constexpr int BI = 64 * WI, BJ = 64 * WJ;
    static constexpr int STAGE_BYTES = (BI + BJ) * 128;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

template <int WI, int WJ>
struct Frags {
    bf16x8 a[WI], b[WJ];
};

template <int WI, int WJ>
__device__ __forceinline__ void mma_block(const Frags<WI, WJ>& f, f32x16 (&acc)[WI][WJ]) {
#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
            acc[ib][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ib], f.b[jb], acc[ib][jb], 0, 0, 0);
}

template <int WI, int WJ>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[WI][WJ]) {
#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.f;
}

// Scheduling hints: spread the LDS fragment reads (and, in the first sub-step, the tile loads of the
// next stage) between the MFMAs instead of in front of them.
template <int N_DS, int N_VMEM, int N_MFMA>
__device__ __forceinline__ void interleave_hint() {
    constexpr int groups = N_DS < N_MFMA ? (N_DS > 0 ? N_DS : 1) : N_MFMA;
    constexpr int mfma_per = N_MFMA / groups;
    constexpr int ds_per = (N_DS + groups - 1) / groups;
    constexpr int vmem_per = (N_VMEM + groups - 1) / groups;
#pragma unroll
    for (int g = 0; g < groups; ++g) {
        if (ds_per > 0) __builtin_amdgcn_sched_group_barrier(0x100, ds_per, 0);       // LDS reads
        if (vmem_per > 0) __builtin_amdgcn_sched_group_barrier(0x010, vmem_per, 0);   // tile loads
        __builtin_amdgcn_sched_group_barrier(0x008, mfma_per, 0);                     // MFMAs
    }
}

__device__ __forceinline__ void dma16(const char* gp, char* lp) {
    // 64 lanes x 16 bytes: lane l's chunk lands at lp + 16 l (lp is wave-uniform)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                     (__attribute__((address_space(3))) void*)lp, 16, 0, 0);
}

// ---------------------------------------------------------------- row-major operands [row][k]
template <int WI, int WJ>
struct RowMajorLoader {
    using S = Shape<WI, WJ>;
    static constexpr int N_DS = WI + WJ;
    static constexpr int N_VMEM = (S::BI + S::BJ) / 32;
    uint32_t voff_a, voff_b;
    int64_t round_a, round_b, wave_a, wave_b;
    int lds_wave_off, a_off, b_off;
    int xo[4];

    __device__ __forceinline__ void init(int64_t lda, int64_t ldb) {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int wave_i = wave & 1, wave_j = wave >> 1;
        // global side: lane l of a wave covers row l/8 of the wave's 8-row band and the chunk that
        // belongs at slot l%8 of that row
        const int gchunk = (lane & 7) ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);
        voff_a = (uint32_t)(((int64_t)(lane >> 3) * lda + gchunk * 8) * 2);
        voff_b = (uint32_t)(((int64_t)(lane >> 3) * ldb + gchunk * 8) * 2);
        wave_a = (int64_t)(wave * 8) * lda * 2;
        wave_b = (int64_t)(wave * 8) * ldb * 2;
        round_a = 32 * lda * 2;
        round_b = 32 * ldb * 2;
        lds_wave_off = wave * 8 * 128;
        // LDS side of the fragment reads
        const int frow = lane & 31, fhi = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) xo[ks] = (((ks * 2 + fhi) ^ ((lane >> 1) & 7)) * 16);
        a_off = (wave_i * (WI * 32) + frow) * 128;
        b_off = S::BI * 128 + (wave_j * (WJ * 32) + frow) * 128;
    }
    __device__ __forceinline__ int64_t step_a() const { return 128; }
    __device__ __forceinline__ int64_t step_b() const { return 128; }
    // ga / gb: wave-uniform byte addresses of the wave's first row at the step's k
    __device__ __forceinline__ void issue(const char* ga, const char* gb, char* stage) const {
#pragma unroll
        for (int t = 0; t < S::BI / 32; ++t) dma16(ga + t * round_a + voff_a, stage + lds_wave_off + t * (32 * 128));
#pragma unroll
        for (int t = 0; t < S::BJ / 32; ++t)
            dma16(gb + t * round_b + voff_b, stage + S::BI * 128 + lds_wave_off + t * (32 * 128));
    }
    __device__ __forceinline__ void frags(Frags<WI, WJ>& f, const char* stage, int ks) const {
#pragma unroll
        for (int ib = 0; ib < WI; ++ib) f.a[ib] = *(const bf16x8*)(stage + a_off + ib * (32 * 128) + xo[ks]);
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) f.b[jb] = *(const bf16x8*)(stage + b_off + jb * (32 * 128) + xo[ks]);
    }
};

// ---------------------------------------------------------------- k-major operands [k][column]
template <int COLS>
struct KMajor {
    static constexpr int ROW_BYTES = COLS * 2;
    static constexpr int CPR = COLS / 8;          // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;          // rows covered by one wave-wide load instruction
    static constexpr int ROUNDS = 64 / (4 * RPI);
    static constexpr int SEGS = CPR / 4;          // 64-byte segments per row
    static constexpr int TILE_BYTES = 64 * ROW_BYTES;
};

__device__ __forceinline__ bf16x8 read_tr_frag(const char* p0, const char* p1) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int WI, int WJ>
struct KMajorLoader {
    using S = Shape<WI, WJ>;
    using KA = KMajor<S::BI>;
    using KB = KMajor<S::BJ>;
    static constexpr int N_DS = 2 * (WI + WJ);
    static constexpr int N_VMEM = KA::ROUNDS + KB::ROUNDS;
    uint32_t voff_a, voff_b;
    int64_t round_a, round_b, wave_a, wave_b, kstep_a, kstep_b;
    int lds_wave_a, lds_wave_b;
    int base_a[2], base_b[2];

    __device__ __forceinline__ void init(int64_t lda, int64_t ldb) {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int wave_i = wave & 1, wave_j = wave >> 1;
        // global side: lane l of a wave instruction covers chunk slot l % CPR of row l / CPR of its band
        {
            const int lrow = lane / KA::CPR, p = lane % KA::CPR;
            const int gseg = (p >> 2) ^ ((wave * KA::RPI + lrow) & (KA::SEGS - 1));
            voff_a = (uint32_t)(((int64_t)lrow * lda + (gseg * 4 + (p & 3)) * 8) * 2);
        }
        {
            const int lrow = lane / KB::CPR, p = lane % KB::CPR;
            const int gseg = (p >> 2) ^ ((wave * KB::RPI + lrow) & (KB::SEGS - 1));
            voff_b = (uint32_t)(((int64_t)lrow * ldb + (gseg * 4 + (p & 3)) * 8) * 2);
        }
        wave_a = (int64_t)(wave * KA::RPI) * lda * 2;
        wave_b = (int64_t)(wave * KB::RPI) * ldb * 2;
        round_a = (int64_t)(4 * KA::RPI) * lda * 2;
        round_b = (int64_t)(4 * KB::RPI) * ldb * 2;
        kstep_a = 64 * lda * 2;
        kstep_b = 64 * ldb * 2;
        lds_wave_a = wave * KA::RPI * KA::ROW_BYTES;
        lds_wave_b = KA::TILE_BYTES + wave * KB::RPI * KB::ROW_BYTES;
        // LDS side: lane l of a transpose read addresses row 8 (l / 32) + (l % 16) / 4 (+ 4 for the
        // second half of the fragment, + 16 per sub-step), 8 bytes at column
        // 32 b + 16 ((l / 16) % 2) + 4 (l % 4) of its block b
        const int q = (lane & 15) >> 2;
        const int sub_bytes = (2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 16 + 8 * (lane & 1);
        const int rowpart = 8 * (lane >> 5) + q;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int sw = 4 * r + q;   // low bits of the row this lane addresses in half r
            base_a[r] = (rowpart + 4 * r) * KA::ROW_BYTES + (((wave_i * WI) ^ (sw & (KA::SEGS - 1))) * 64) + sub_bytes;
            base_b[r] = KA::TILE_BYTES + (rowpart + 4 * r) * KB::ROW_BYTES +
                        (((wave_j * WJ) ^ (sw & (KB::SEGS - 1))) * 64) + sub_bytes;
        }
    }
    __device__ __forceinline__ int64_t step_a() const { return kstep_a; }
    __device__ __forceinline__ int64_t step_b() const { return kstep_b; }
    __device__ __forceinline__ void issue(const char* ga, const char* gb, char* stage) const {
#pragma unroll
        for (int t = 0; t < KA::ROUNDS; ++t)
            dma16(ga + t * round_a + voff_a, stage + lds_wave_a + t * (4 * KA::RPI * KA::ROW_BYTES));
#pragma unroll
        for (int t = 0; t < KB::ROUNDS; ++t)
            dma16(gb + t * round_b + voff_b, stage + lds_wave_b + t * (4 * KB::RPI * KB::ROW_BYTES));
    }
    __device__ __forceinline__ void frags(Frags<WI, WJ>& f, const char* stage, int ks) const {
        // the block index b enters the swizzled segment by XOR (blocks per wave are a power of two)
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
            f.a[ib] = read_tr_frag(stage + ks * 16 * KA::ROW_BYTES + (base_a[0] ^ (ib * 64)),
                                   stage + ks * 16 * KA::ROW_BYTES + (base_a[1] ^ (ib * 64)));
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
            f.b[jb] = read_tr_frag(stage + ks * 16 * KB::ROW_BYTES + (base_b[0] ^ (jb * 64)),
                                   stage + ks * 16 * KB::ROW_BYTES + (base_b[1] ^ (jb * 64)));
    }
};

// ---------------------------------------------------------------- tile schedule of a workgroup
struct Sched {
    int first, stride, count;
};
__device__ __forceinline__ Sched make_sched(int total) {
    const int nwg = gridDim.x, w = blockIdx.x;
    const int xcd = w & 7, slot = w >> 3, nslot = nwg >> 3;
    const int per = (total + 7) >> 3;
    const int lo = xcd * per;
    const int hi = min(lo + per, total);
    Sched s;
    s.first = lo + slot;
    s.stride = nslot;
    s.count = s.first < hi ? (hi - s.first + nslot - 1) / nslot : 0;
    return s;
}
// grouped order: GI tiles along i for one j, then the next j, ...
struct TileCoord {
    int ti, tj;
};
__device__ __forceinline__ TileCoord map_tile(int vid, int tilesI, int tilesJ, int GI) {
    const int group_sz = GI * tilesJ;
    const int grp = vid / group_sz;
    const int first_i = grp * GI;
    const int gi = min(GI, tilesI - first_i);
    const int rem = vid - grp * group_sz;
    TileCoord t;
    t.ti = first_i + rem % gi;
    t.tj = rem / gi;
    return t;
}

// Runs this workgroup's tiles.  tile(vid, A, B, coord) gives the operand addresses of a tile (first
// row, k = 0); epi(coord, acc) consumes a finished accumulator tile.
template <int WI, int WJ, class Loader, class TileFn, class EpiFn>
__device__ __forceinline__ void run_tiles(Loader& ld, char* lds, const Sched& sch, int ktiles, TileFn&& tile,
                                          EpiFn&& epi, int dbg = 0) {
    using S = Shape<WI, WJ>;
    f32x16 acc[WI][WJ];
    zero_acc<WI, WJ>(acc);
    if (sch.count <= 0) return;
    if (ktiles <= 0) {   // empty contraction: the tiles are zero
        for (int n = 0; n < sch.count; ++n) {
            const bf16_t *A, *B;
            TileCoord c;
            tile(sch.first + n * sch.stride, A, B, c);
            epi(c, acc);
        }
        return;
    }
    const bf16_t *A, *B;
    TileCoord cur_c, next_c;
    tile(sch.first, A, B, cur_c);
    const char* ga = (const char*)A + ld.wave_a;
    const char* gb = (const char*)B + ld.wave_b;
    ld.issue(ga, gb, lds);
    int parity = 0;
    Frags<WI, WJ> f0, f1;
    for (int n = 0; n < sch.count; ++n) {
        // where the loads go after this tile's last step: the next tile, or (for the last tile) this
        // tile's first step again, which is in bounds and never consumed
        const int next_vid = sch.first + (n + 1 < sch.count ? n + 1 : n) * sch.stride;
        tile(next_vid, A, B, next_c);
        const char* nga = (const char*)A + ld.wave_a;
        const char* ngb = (const char*)B + ld.wave_b;
        for (int kt = 0; kt < ktiles; ++kt) {
            char* cur = lds + parity * S::STAGE_BYTES;
            char* nxt = lds + (parity ^ 1) * S::STAGE_BYTES;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();   // stage `cur` has landed for every wave; nobody still reads `nxt`
            const bool last = kt + 1 == ktiles;
            ga = last ? nga : ga + ld.step_a();
            gb = last ? ngb : gb + ld.step_b();
            if (dbg & 1) {   // timing experiment: tile loads only
                ld.issue(ga, gb, nxt);
                parity ^= 1;
                continue;
            }
            ld.frags(f0, cur, 0);
            if (!(dbg & 2)) ld.issue(ga, gb, nxt);
            ld.frags(f1, cur, 1);
            mma_block<WI, WJ>(f0, acc);
            interleave_hint<Loader::N_DS, Loader::N_VMEM, WI * WJ>();
            ld.frags(f0, cur, 2);
            mma_block<WI, WJ>(f1, acc);
            interleave_hint<Loader::N_DS, 0, WI * WJ>();
            ld.frags(f1, cur, 3);
            mma_block<WI, WJ>(f0, acc);
            interleave_hint<Loader::N_DS, 0, WI * WJ>();
            mma_block<WI, WJ>(f1, acc);
            parity ^= 1;
        }
        epi(cur_c, acc);
        zero_acc<WI, WJ>(acc);
        cur_c = next_c;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the spare load of the last step
}

struct Lane {
    int lane, wave_i, wave_j, hi, lj;
    __device__ __forceinline__ Lane() {
        lane = threadIdx.x & 63;
        const int w = threadIdx.x >> 6;
        wave_i = w & 1;
        wave_j = w >> 1;
        hi = lane >> 5;
        lj = lane & 31;
    }
};

__device__ __forceinline__ uint2 pack_bf16x4(float a, float b, float c, float d) {
    bf16x4 r;
    r[0] = (__bf16)a; r[1] = (__bf16)b; r[2] = (__bf16)c; r[3] = (__bf16)d;
    return __builtin_bit_cast(uint2, r);
}

// ------------------------------------------------------------------------------------- fwd_lse
template <int WI, int WJ>
__global__ __launch_bounds__(NT) void fwd_lse_kernel(FwdArgs a) {
    using S = Shape<WI, WJ>;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesM = a.counts[CNT_MR] / S::BJ;   // row tiles that hold tokens
    const Sched sch = make_sched(a.tilesV * tilesM);
    RowMajorLoader<WI, WJ> ld;
    ld.init(a.ldk, a.ldk);
    const Lane L;
    auto tile = [&](int vid, const bf16_t*& A, const bf16_t*& B, TileCoord& c) {
        c = map_tile(vid, a.tilesV, tilesM, 4);
        A = a.Wvd + (int64_t)c.ti * S::BI * a.ldk;
        B = a.Hc + (int64_t)c.tj * S::BJ * a.ldk;
    };
    auto epi = [&](const TileCoord& t, f32x16 (&acc)[WI][WJ]) {
        const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
        const bool tail = i_base + WI * 32 > a.V;
        const int64_t slot = (int64_t)t.ti * 2 + L.wave_i;
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) {
            const int64_t j = (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
            const int tok = a.tokc[j];
            float m = -INFINITY, zyv = 0.f;
            bool found = false;
#pragma unroll
            for (int ib = 0; ib < WI; ++ib)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t i = i_base + ib * 32 + (v >> 2) * 8 + L.hi * 4 + (v & 3);
                    float z = acc[ib][jb][v] * a.inv_temp;
                    if (tail && i >= a.V) z = -INFINITY;
                    acc[ib][jb][v] = z;
                    m = fmaxf(m, z);
                    if (i == tok) { zyv = z; found = true; }
                }
            m = fmaxf(m, __shfl_xor(m, 32, 64));
            const float mm = (m == -INFINITY) ? 0.f : m;
            float l = 0.f;
#pragma unroll
            for (int ib = 0; ib < WI; ++ib)
#pragma unroll
                for (int v = 0; v < 16; ++v) l += __builtin_amdgcn_exp2f((acc[ib][jb][v] - mm) * LOG2E);
            l += __shfl_xor(l, 32, 64);
            if (L.hi == 0) {
                a.part_max[slot * a.ld_part + j] = m;
                a.part_sum[slot * a.ld_part + j] = l;
            }
            if (found) a.zy[j] = zyv;
        }
    };
    run_tiles<WI, WJ>(ld, lds, sch, (int)(a.dpad / K_TILE), tile, epi, a.dbg);
}

// ------------------------------------------------------------------------------------------ dz
template <int WI, int WJ>
__global__ __launch_bounds__(NT) void dz_kernel(DzArgs a) {
    using S = Shape<WI, WJ>;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    int64_t rows = (int64_t)Mr - a.m0;
    rows = rows < 0 ? 0 : (rows > (int64_t)a.tilesM * S::BJ ? (int64_t)a.tilesM * S::BJ : rows);
    const int tilesM = (int)(rows / S::BJ);
    const Sched sch = make_sched(a.tilesV * tilesM);
    RowMajorLoader<WI, WJ> ld;
    ld.init(a.ldk, a.ldk);
    const Lane L;
    auto tile = [&](int vid, const bf16_t*& A, const bf16_t*& B, TileCoord& c) {
        c = map_tile(vid, a.tilesV, tilesM, 4);
        A = a.Wvd + (int64_t)c.ti * S::BI * a.ldk;
        B = a.Hc + (int64_t)c.tj * S::BJ * a.ldk;
    };
    auto epi = [&](const TileCoord& t, f32x16 (&acc)[WI][WJ]) {
        const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
        const float zs = a.inv_temp * LOG2E;
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) {
            const int64_t jl = (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;   // row in chunk
            const int64_t j = a.m0 + jl;
            const bool live = j < M;
            const int tok = a.tokc[j];
            const float gj = live ? a.g[a.seqc[j]] * a.inv_temp : 0.f;
            const float nlse = live ? -a.lse_c[j] * LOG2E : 0.f;
            bf16_t* out = a.dz + jl * a.ldz;
#pragma unroll
            for (int ib = 0; ib < WI; ++ib)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t i0 = i_base + ib * 32 + q * 8 + L.hi * 4;
                    float o[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int64_t i = i0 + r;
                        const float p = __builtin_amdgcn_exp2f(fmaf(acc[ib][jb][q * 4 + r], zs, nlse));
                        float val = gj * ((i == tok ? 1.f : 0.f) - p);
                        if (!live || i >= a.V) val = 0.f;
                        o[r] = val;
                    }
                    *(uint2*)(out + i0) = pack_bf16x4(o[0], o[1], o[2], o[3]);
                }
        }
    };
    run_tiles<WI, WJ>(ld, lds, sch, (int)(a.dpad / K_TILE), tile, epi, a.dbg);
}

// ------------------------------------------------------------------------------------------ dh
template <int WI, int WJ>
__global__ __launch_bounds__(NT) void dh_kernel(DhArgs a) {
    using S = Shape<WI, WJ>;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesD = (int)(a.dpadR / S::BI);
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    int64_t rows = (int64_t)Mr - a.m0;
    rows = rows < 0 ? 0 : (rows > (int64_t)a.tilesM * S::BJ ? (int64_t)a.tilesM * S::BJ : rows);
    const int tilesM = (int)(rows / S::BJ);
    const Sched sch = make_sched(tilesD * tilesM);
    RowMajorLoader<WI, WJ> ld;
    ld.init(a.ldv, a.ldv);
    const Lane L;
    auto tile = [&](int vid, const bf16_t*& A, const bf16_t*& B, TileCoord& c) {
        c = map_tile(vid, tilesD, tilesM, tilesD);
        A = a.Wdv + (int64_t)c.ti * S::BI * a.ldv;
        B = a.dz + (int64_t)c.tj * S::BJ * a.ldv;
    };
    auto epi = [&](const TileCoord& t, f32x16 (&acc)[WI][WJ]) {
        const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) {
            const int64_t j = a.m0 + (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
            if (j >= M) continue;
            bf16_t* out = a.dhidden + (int64_t)a.row_index[j] * a.d;
#pragma unroll
            for (int ib = 0; ib < WI; ++ib)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t i0 = i_base + ib * 32 + q * 8 + L.hi * 4;
                    if (i0 < a.d)
                        *(uint2*)(out + i0) = pack_bf16x4(acc[ib][jb][q * 4], acc[ib][jb][q * 4 + 1],
                                                          acc[ib][jb][q * 4 + 2], acc[ib][jb][q * 4 + 3]);
                }
        }
    };
    run_tiles<WI, WJ>(ld, lds, sch, (int)(a.Vpad / K_TILE), tile, epi, a.dbg);
}

// ------------------------------------------------------------------------------------------ dw
template <int WI, int WJ>
__global__ __launch_bounds__(NT) void dw_kernel(DwArgs a) {
    using S = Shape<WI, WJ>;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesV = (int)(a.Vpad / S::BI), tilesD = (int)(a.dpadR / S::BJ);
    const int Mr = a.counts[CNT_MR];
    int64_t rows = (int64_t)Mr - a.m0;
    rows = rows < 0 ? 0 : (rows > a.Mc ? a.Mc : rows);
    if (rows == 0 && a.beta) return;   // nothing to add
    const Sched sch = make_sched(tilesV * tilesD);
    KMajorLoader<WI, WJ> ld;
    ld.init(a.ldz, a.ldH);
    const Lane L;
    auto tile = [&](int vid, const bf16_t*& A, const bf16_t*& B, TileCoord& c) {
        c = map_tile(vid, tilesV, tilesD, 8);
        A = a.dz + (int64_t)c.ti * S::BI;
        B = a.Hc + (int64_t)c.tj * S::BJ;
    };
    const bool vec = (a.V % 4) == 0;
    auto epi = [&](const TileCoord& t, f32x16 (&acc)[WI][WJ]) {
        const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) {
            const int64_t jd = (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
            if (jd >= a.d) continue;
#pragma unroll
            for (int ib = 0; ib < WI; ++ib)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t i0 = i_base + ib * 32 + q * 8 + L.hi * 4;
                    if (i0 >= a.V) continue;
                    float o[4] = {acc[ib][jb][q * 4], acc[ib][jb][q * 4 + 1], acc[ib][jb][q * 4 + 2],
                                  acc[ib][jb][q * 4 + 3]};
                    if (a.w_layout == RAPID_W_DV) {
                        float* p = a.dW + jd * a.V + i0;
                        if (vec) {
                            float4 cur = make_float4(0.f, 0.f, 0.f, 0.f);
                            if (a.beta) cur = *(const float4*)p;
                            *(float4*)p = make_float4(cur.x + o[0], cur.y + o[1], cur.z + o[2], cur.w + o[3]);
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (i0 + r < a.V) p[r] = (a.beta ? p[r] : 0.f) + o[r];
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (i0 + r < a.V) {
                                float* p = a.dW + (i0 + r) * a.d + jd;
                                *p = (a.beta ? *p : 0.f) + o[r];
                            }
                    }
                }
        }
    };
    run_tiles<WI, WJ>(ld, lds, sch, (int)(rows / K_TILE), tile, epi, a.dbg);
}

template <class K>
void allow_lds(K kernel, int bytes) {
    (void)hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// one workgroup per CU, a multiple of 8 so that every XCD gets the same number
unsigned persistent_grid() {
    static int cached = 0;
    if (!cached) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
            cus = 256;
        cached = cus / 8 * 8;
    }
    return (unsigned)cached;
}

}  // namespace

void launch_fwd_lse(const FwdArgs& a, hipStream_t st) {
    using S = Shape<4, 4>;
    allow_lds(fwd_lse_kernel<4, 4>, S::LDS_BYTES);
    fwd_lse_kernel<4, 4><<<persistent_grid(), NT, S::LDS_BYTES, st>>>(a);
}
int fwd_slots_per_tile() { return 2; }

void launch_dz(const DzArgs& a, hipStream_t st) {
    using S = Shape<4, 4>;
    allow_lds(dz_kernel<4, 4>, S::LDS_BYTES);
    dz_kernel<4, 4><<<persistent_grid(), NT, S::LDS_BYTES, st>>>(a);
}

void launch_dh(const DhArgs& a, hipStream_t st) {
    if (a.dpadR % 256 == 0) {
        using S = Shape<4, 4>;
        allow_lds(dh_kernel<4, 4>, S::LDS_BYTES);
        dh_kernel<4, 4><<<persistent_grid(), NT, S::LDS_BYTES, st>>>(a);
    } else {   // d padded to a multiple of 128 only
        using S = Shape<2, 4>;
        allow_lds(dh_kernel<2, 4>, S::LDS_BYTES);
        dh_kernel<2, 4><<<persistent_grid(), NT, S::LDS_BYTES, st>>>(a);
    }
}

void launch_dw(const DwArgs& a, hipStream_t st) {
    if (a.dpadR % 256 == 0) {
        using S = Shape<4, 4>;
        allow_lds(dw_kernel<4, 4>, S::LDS_BYTES);
        dw_kernel<4, 4><<<persistent_grid(), NT, S::LDS_BYTES, st>>>(a);
    } else {
        using S = Shape<4, 2>;
        allow_lds(dw_kernel<4, 2>, S::LDS_BYTES);
        dw_kernel<4, 2><<<persistent_grid(), NT, S::LDS_BYTES, st>>>(a);
    }
}

}  // namespace rapid
