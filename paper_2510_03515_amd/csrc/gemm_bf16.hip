// bf16 MFMA contractions of the hot path for gfx950 (CDNA4): one tiled main loop (two operand
// layouts) and four epilogues.
//   fwd_lse : logits tile  -> per-slot (max, sum exp) of the streaming log-softmax + gathered logit
//   dz      : logits tile  -> dz = g (onehot - softmax) / temperature, written as bf16
//   dh      : dH = dz . W^T          (contraction over the vocabulary)
//   dw      : dW (+)= H^T . dz       (contraction over the tokens of a row chunk)
//
// Tiling.  C[i][j] = sum_k A(i,k) B(j,k); operands are zero padded to whole tiles, so the loop has
// no bounds checks.  A workgroup of four 64-lane waves (2 x 2) owns a (64 WI) x (64 WJ) tile, each
// wave WI x WJ blocks of 32 x 32 computed with v_mfma_f32_32x32x16_bf16 (a lane feeds 8 consecutive
// k of one row).  The 256 x 256 tile fills the register file (256 accumulator registers per lane)
// and is the largest a CU can hold, which minimises L2 -> LDS bytes per flop.  K advances 64
// elements per step through two LDS stages of 64 KiB (one barrier per step); operand tiles arrive
// by global_load_lds_dwordx4 (memory -> LDS without passing through registers; consecutive lanes
// fill consecutive 16-byte slots, so the LDS swizzle is applied to the global address).  One
// workgroup computes one tile; workgroup ids are mapped to tiles so that the workgroups resident
// on an XCD (ids equal mod 8) own neighbouring tiles and share operand panels in that XCD's L2.
//
// LDS layouts (both conflict-free for a 256-byte LDS cycle, checked with SQ_LDS_BANK_CONFLICT):
//  * row-major operands ([row][k], k contiguous): a tile row of a step is 128 bytes = 8 chunks of
//    16 bytes; chunk c of row r sits at position c ^ ((r >> 1) & 7); fragments are read with
//    ds_read_b128.
//  * k-major operands ([k][column], used by dW where the contraction index is the token row): see
//    the comment above KMajor below; fragments are read with the LDS transpose read.
//
// Accumulator layout of a 32 x 32 block (lane l, register v): j = l % 32,
// i = 8 (v / 4) + 4 (l / 32) + v % 4: a lane owns runs of 4 consecutive i for one j, so every
// epilogue keeps j = the token row (per-lane scalars: lse, coefficient, token id, output row) and
// stores 4 consecutive i with one 8- or 16-byte access.
#include "rapid_internal.h"

namespace rapid {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float LOG2E = 1.4426950408889634f;

// Geometry of a workgroup: NWI x NWJ waves, each owning WI x WJ blocks of 32 x 32.
// Two are used: 2 x 2 waves of 128 x 128 (one wave per SIMD, 256 accumulator registers per lane) and
// 2 x 4 waves of 128 x 64 (two waves per SIMD, which lets the hardware overlap one wave's LDS and
// barrier waits with the other's MFMAs at the price of 1.5x the LDS fragment reads).
template <int NWI_, int NWJ_, int WI_, int WJ_>
struct Geo {
    static constexpr int NWI = NWI_, NWJ = NWJ_, WI = WI_, WJ = WJ_;
    static constexpr int NW = NWI * NWJ, NT = 64 * NW;
    static constexpr int BI = NWI * WI * 32, BJ = NWJ * WJ * 32;
    static constexpr int STAGE_BYTES = (BI + BJ) * 128;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

__device__ __forceinline__ void lds_barrier() { __syncthreads(); }

// Requests one K step (64 columns) of a tile with ROWS rows: direct memory -> LDS loads, 16 bytes
// per lane.  `gwave` is the wave-uniform address of the wave's first row of round 0 (scalar
// registers), `voff` the lane's byte offset from it (row lane/8 of the 8-row band, swizzled chunk),
// `round_bytes` the uniform distance between rounds (8 rows per wave); lane l's chunk lands at
// lds_wave + 16 l of each round.
template <int ROWS, int NW>
__device__ __forceinline__ void issue_tile_load(const char* __restrict__ gwave, uint32_t voff, int64_t round_bytes,
                                                char* lds_wave) {
#pragma unroll
    for (int t = 0; t < ROWS / (8 * NW); ++t)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gwave + t * round_bytes + voff),
                                         (__attribute__((address_space(3))) void*)(lds_wave + t * (8 * NW * 128)), 16, 0, 0);
}

template <int WI, int WJ>
struct Frags {
    bf16x8 a[WI], b[WJ];
};

template <int WI, int WJ>
__device__ __forceinline__ void load_frags(Frags<WI, WJ>& f, const char* cur, int a_off, int b_off, int xo) {
#pragma unroll
    for (int ib = 0; ib < WI; ++ib) f.a[ib] = *(const bf16x8*)(cur + a_off + ib * (32 * 128) + xo);
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) f.b[jb] = *(const bf16x8*)(cur + b_off + jb * (32 * 128) + xo);
}

template <int WI, int WJ>
__device__ __forceinline__ void mma_block(const Frags<WI, WJ>& f, f32x16 (&acc)[WI][WJ]) {
#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
            acc[ib][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ib], f.b[jb], acc[ib][jb], 0, 0, 0);
}

// Scheduling hints: keep the matrix pipe fed by spreading the LDS fragment reads (and, in the
// first sub-step, the tile loads of the next stage) between the MFMAs instead of in front of them.
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

// acc += A_tile . B_tile^T over `ktiles` steps of 64.  A / B point at the tile's first row, k = 0.
template <class S>
__device__ __forceinline__ void mainloop(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                                         int64_t ldb, int ktiles, char* lds, f32x16 (&acc)[S::WI][S::WJ]) {
    constexpr int WI = S::WI, WJ = S::WJ;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_i = wave % S::NWI, wave_j = wave / S::NWI;

    // global side of the tile loads: lane l of a wave covers row l/8 of the wave's 8-row band and
    // the chunk that belongs at slot l%8 of that row
    const int gchunk = (lane & 7) ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);
    const uint32_t voff_a = (uint32_t)(((int64_t)(lane >> 3) * lda + gchunk * 8) * 2);
    const uint32_t voff_b = (uint32_t)(((int64_t)(lane >> 3) * ldb + gchunk * 8) * 2);
    const char* ga = (const char*)(A + (int64_t)(wave * 8) * lda);
    const char* gb = (const char*)(B + (int64_t)(wave * 8) * ldb);
    const int64_t round_a = (8 * S::NW) * lda * 2, round_b = (8 * S::NW) * ldb * 2;
    const int lds_wave_off = wave * 8 * 128;

    // LDS side of the fragment reads
    const int frow = lane & 31, fhi = lane >> 5;
    int xo[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) xo[ks] = (((ks * 2 + fhi) ^ ((lane >> 1) & 7)) * 16);
    const int a_off = (wave_i * (WI * 32) + frow) * 128;
    const int b_off = S::BI * 128 + (wave_j * (WJ * 32) + frow) * 128;

#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.f;

    if (ktiles <= 0) return;

    issue_tile_load<S::BI, S::NW>(ga, voff_a, round_a, lds + lds_wave_off);
    issue_tile_load<S::BJ, S::NW>(gb, voff_b, round_b, lds + S::BI * 128 + lds_wave_off);

    Frags<WI, WJ> f0, f1;
    for (int kt = 0; kt < ktiles; ++kt) {
        char* cur = lds + (kt & 1) * S::STAGE_BYTES;
        char* nxt = lds + ((kt + 1) & 1) * S::STAGE_BYTES;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();   // stage `cur` is complete; nobody still reads stage `nxt`
        // the last step re-loads its own tile into the idle stage, which keeps the loop body free
        // of branches (one scheduling region) and every address in bounds
        const int adv = (kt + 1 < ktiles) ? 128 : 0;
        ga += adv;
        gb += adv;
        load_frags<WI, WJ>(f0, cur, a_off, b_off, xo[0]);
        issue_tile_load<S::BI, S::NW>(ga, voff_a, round_a, nxt + lds_wave_off);
        issue_tile_load<S::BJ, S::NW>(gb, voff_b, round_b, nxt + S::BI * 128 + lds_wave_off);
        load_frags<WI, WJ>(f1, cur, a_off, b_off, xo[1]);
        mma_block<WI, WJ>(f0, acc);
        interleave_hint<WI + WJ, (S::BI + S::BJ) / (8 * S::NW), WI * WJ>();
        load_frags<WI, WJ>(f0, cur, a_off, b_off, xo[2]);
        mma_block<WI, WJ>(f1, acc);
        interleave_hint<WI + WJ, 0, WI * WJ>();
        load_frags<WI, WJ>(f1, cur, a_off, b_off, xo[3]);
        mma_block<WI, WJ>(f0, acc);
        interleave_hint<WI + WJ, 0, WI * WJ>();
        mma_block<WI, WJ>(f1, acc);
    }
}

// ---- contraction index major operands ("k-major") ---------------------------------------------
// For dW = H^T dz both operands are stored with the contraction index (the token row) as the slow
// dimension: A(k, i) = dz[row k][column i], B(k, j) = H[row k][column j].  A K step is 64 rows of
// 2 COLS bytes; it goes to LDS row by row (direct loads, 16-byte chunks) and the MFMA fragments are
// read with ds_read_b64_tr_b16, the LDS transpose read of gfx950: in each group of 16 lanes, lane
// l receives element (l % 4) of the 8-byte pieces addressed by lanes l/4, l/4 + 4, l/4 + 8,
// l/4 + 12 of the group.  Pointing lane s of a group at row (s / 4), columns 4 (s % 4) .. + 3
// therefore hands lane l column l and 4 consecutive rows: exactly the per-lane slice of an MFMA
// operand (row of the operand = column of the tile, 4 of its 8 k values).
// A row is cut into 64-byte segments and segment g of row r is kept at position g ^ (r % SEGS),
// so that the four rows one transpose read touches per 32 lanes fall on different banks.
template <int COLS, int NW>
struct KMajor {
    static constexpr int ROW_BYTES = COLS * 2;
    static constexpr int CPR = COLS / 8;          // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;          // rows covered by one wave-wide load instruction
    static constexpr int ROUNDS = 64 / (NW * RPI);
    static constexpr int ROUND_ROWS = NW * RPI;
    static constexpr int SEGS = CPR / 4;          // 64-byte segments per row
    static constexpr int TILE_BYTES = 64 * ROW_BYTES;
};

template <int COLS, int NW>
__device__ __forceinline__ void issue_kmajor_load(const char* __restrict__ gwave, uint32_t voff, int64_t round_bytes,
                                                  char* lds_wave) {
    using KM = KMajor<COLS, NW>;
#pragma unroll
    for (int t = 0; t < KM::ROUNDS; ++t) {
        const char* gp = gwave + t * round_bytes + voff;
        char* lp = lds_wave + t * (KM::ROUND_ROWS * KM::ROW_BYTES);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                         (__attribute__((address_space(3))) void*)lp, 16, 0, 0);
    }
}

typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 read_tr_frag(const char* p0, const char* p1) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// acc[i-block][j-block] += sum over `ktiles` steps of 64 rows of A(k, i) B(k, j).
// A points at (row 0, first column of the i tile), B likewise; lda / ldb are row strides in elements.
template <class S>
__device__ __forceinline__ void mainloop_kmajor(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                                                int64_t ldb, int ktiles, char* lds, f32x16 (&acc)[S::WI][S::WJ]) {
    constexpr int WI = S::WI, WJ = S::WJ;
    using KA = KMajor<S::BI, S::NW>;
    using KB = KMajor<S::BJ, S::NW>;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_i = wave % S::NWI, wave_j = wave / S::NWI;

    // global side: lane l of a wave instruction covers chunk slot l % CPR of row l / CPR of its band
    auto lane_voff = [&](int cpr, int segs, int rpi, int64_t ld) -> uint32_t {
        const int lrow = lane / cpr, p = lane % cpr;
        const int row_low = (wave * rpi + lrow) & (segs - 1);
        const int gseg = (p >> 2) ^ row_low;
        return (uint32_t)(((int64_t)lrow * ld + (gseg * 4 + (p & 3)) * 8) * 2);
    };
    const uint32_t voff_a = lane_voff(KA::CPR, KA::SEGS, KA::RPI, lda);
    const uint32_t voff_b = lane_voff(KB::CPR, KB::SEGS, KB::RPI, ldb);
    const char* ga = (const char*)(A + (int64_t)(wave * KA::RPI) * lda);
    const char* gb = (const char*)(B + (int64_t)(wave * KB::RPI) * ldb);
    const int64_t round_a = (int64_t)KA::ROUND_ROWS * lda * 2, round_b = (int64_t)KB::ROUND_ROWS * ldb * 2;
    const int64_t step_a = 64 * lda * 2, step_b = 64 * ldb * 2;
    const int lds_wave_a = wave * KA::RPI * KA::ROW_BYTES;
    const int lds_wave_b = KA::TILE_BYTES + wave * KB::RPI * KB::ROW_BYTES;

    // LDS side: lane l of a transpose read addresses row 8 (l / 32) + (l % 16) / 4 (+ 4 for the second
    // half of the fragment, + 16 per sub-step), 8 bytes at column 32 b + 16 ((l / 16) % 2) + 4 (l % 4)
    const int q = (lane & 15) >> 2;
    const int sub_bytes = (2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 16 + 8 * (lane & 1);
    const int rowpart = 8 * (lane >> 5) + q;
    int base_a[2], base_b[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int sw = 4 * r + q;   // low bits of the row this lane addresses in half r
        base_a[r] = (rowpart + 4 * r) * KA::ROW_BYTES + ((((wave_i * WI) ^ (sw & (KA::SEGS - 1))) * 64)) + sub_bytes;
        base_b[r] = KA::TILE_BYTES + (rowpart + 4 * r) * KB::ROW_BYTES +
                    ((((wave_j * WJ) ^ (sw & (KB::SEGS - 1))) * 64)) + sub_bytes;
    }

    auto load_frags_t = [&](Frags<WI, WJ>& f, const char* cur, int ks) {
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
            f.a[ib] = read_tr_frag(cur + ks * 16 * KA::ROW_BYTES + (base_a[0] ^ (ib * 64)),
                                   cur + ks * 16 * KA::ROW_BYTES + (base_a[1] ^ (ib * 64)));
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
            f.b[jb] = read_tr_frag(cur + ks * 16 * KB::ROW_BYTES + (base_b[0] ^ (jb * 64)),
                                   cur + ks * 16 * KB::ROW_BYTES + (base_b[1] ^ (jb * 64)));
    };

#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.f;

    if (ktiles <= 0) return;

    issue_kmajor_load<S::BI, S::NW>(ga, voff_a, round_a, lds + lds_wave_a);
    issue_kmajor_load<S::BJ, S::NW>(gb, voff_b, round_b, lds + lds_wave_b);

    Frags<WI, WJ> f0, f1;
    for (int kt = 0; kt < ktiles; ++kt) {
        char* cur = lds + (kt & 1) * S::STAGE_BYTES;
        char* nxt = lds + ((kt + 1) & 1) * S::STAGE_BYTES;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        const bool more = kt + 1 < ktiles;   // the last step re-loads its own rows into the idle stage
        ga += more ? step_a : 0;
        gb += more ? step_b : 0;
        load_frags_t(f0, cur, 0);
        issue_kmajor_load<S::BI, S::NW>(ga, voff_a, round_a, nxt + lds_wave_a);
        issue_kmajor_load<S::BJ, S::NW>(gb, voff_b, round_b, nxt + lds_wave_b);
        load_frags_t(f1, cur, 1);
        mma_block<WI, WJ>(f0, acc);
        interleave_hint<2 * (WI + WJ), KA::ROUNDS + KB::ROUNDS, WI * WJ>();
        load_frags_t(f0, cur, 2);
        mma_block<WI, WJ>(f1, acc);
        interleave_hint<2 * (WI + WJ), 0, WI * WJ>();
        load_frags_t(f1, cur, 3);
        mma_block<WI, WJ>(f0, acc);
        interleave_hint<2 * (WI + WJ), 0, WI * WJ>();
        mma_block<WI, WJ>(f1, acc);
    }
}

// Workgroup id -> tile.  Hardware deals consecutive workgroup ids round-robin to the 8 XCDs (each
// with its own L2), so id % 8 picks the XCD and id / 8 the position in that XCD's contiguous share
// of a grouped order: GI tiles along i for one j, then the next j, ... so that workgroups resident
// together on an XCD re-use each other's operand panels out of L2.
struct TileId { int ti, tj; bool valid; };
__device__ __forceinline__ TileId map_tile(int pid, int tilesI, int tilesJ, int GI) {
    const int total = tilesI * tilesJ;
    const int per = (total + 7) / 8;
    const int vid = (pid & 7) * per + (pid >> 3);
    TileId t;
    t.valid = vid < total;
    const int group_sz = GI * tilesJ;
    const int grp = vid / group_sz;
    const int first_i = grp * GI;
    const int gi = min(GI, tilesI - first_i);
    const int rem = vid - grp * group_sz;
    t.ti = first_i + rem % gi;
    t.tj = rem / gi;
    return t;
}
inline unsigned grid_for(int tilesI, int tilesJ) { return (unsigned)(((int64_t)tilesI * tilesJ + 7) / 8 * 8); }

template <class S>
struct Lane {
    int lane, wave, wave_i, wave_j, hi, lj;
    __device__ __forceinline__ Lane() {
        lane = threadIdx.x & 63;
        wave = threadIdx.x >> 6;
        wave_i = wave % S::NWI;
        wave_j = wave / S::NWI;
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
template <class S>
__global__ __launch_bounds__(S::NT) void fwd_lse_kernel(FwdArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const TileId t = map_tile(blockIdx.x, a.tilesV, a.tilesM, a.gi);
    if (!t.valid) return;
    const int Mr = a.counts[CNT_MR];
    if ((int64_t)t.tj * S::BJ >= Mr) return;
    f32x16 acc[WI][WJ];
    mainloop<S>(a.Wvd + (int64_t)t.ti * S::BI * a.ldk, a.ldk,
                             a.Hc + (int64_t)t.tj * S::BJ * a.ldk, a.ldk, (int)(a.dpad / K_TILE), lds, acc);
    // Epilogue: per token row j (one lane pair) the max and the sum of exponentials over this wave's
    // 128 vocabulary columns.  The logit of the sampled token is gathered by a separate small kernel,
    // so the per-element work is one max, one fma, one exp and one add.
    const Lane<S> L;
    const int i_base = t.ti * S::BI + L.wave_i * (WI * 32);
    const int n_valid = (int)a.V - i_base;          // columns of this wave that exist (>= 128: all)
    const int64_t slot = (int64_t)t.ti * S::NWI + L.wave_i;
    const float zs = a.inv_temp * LOG2E;            // inv_temp > 0: max commutes with the scaling
    if (n_valid < WI * 32) {                        // ragged last vocabulary tile: mask the padding
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rel = ib * 32 + (v >> 2) * 8 + L.hi * 4 + (v & 3);
                    acc[ib][jb][v] = rel < n_valid ? acc[ib][jb][v] : -INFINITY;
                }
    }
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int64_t j = (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
        float m = -INFINITY;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) m = fmaxf(m, acc[ib][jb][v]);
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        const float nm = (m == -INFINITY) ? 0.f : -m * zs;
        float l = 0.f;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) l += __builtin_amdgcn_exp2f(fmaf(acc[ib][jb][v], zs, nm));
        l += __shfl_xor(l, 32, 64);
        if (L.hi == 0) {
            a.part_max[slot * a.ld_part + j] = m * a.inv_temp;
            a.part_sum[slot * a.ld_part + j] = l;
        }
    }
}

// ------------------------------------------------------------------------------------------ dz
// Epilogue: the tile leaves through LDS so that it reaches memory as whole 256-byte row segments.
// Each wave owns a private 32 KiB region (its 128 rows x 128 columns of bf16, 256 bytes per row;
// the four regions are exactly the two idle LDS stages).  A lane writes its runs of 4 consecutive
// columns (8 bytes) at 16-byte chunk c ^ (row % 16) of the row, then the wave reads the region
// back row-wise, 16 lanes x 16 bytes per row, and stores 4 full rows per instruction.
template <class S>
__global__ __launch_bounds__(S::NT) void dz_kernel(DzArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    static_assert(WI == 4, "the LDS-staged epilogue is laid out for 128 columns (256 bytes) per wave row");
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const TileId t = map_tile(blockIdx.x, a.tilesV, a.tilesM, a.gi);
    if (!t.valid) return;
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.m0 + (int64_t)t.tj * S::BJ >= Mr) return;
    f32x16 acc[WI][WJ];
    mainloop<S>(a.Wvd + (int64_t)t.ti * S::BI * a.ldk, a.ldk,
                     a.Hc + (int64_t)t.tj * S::BJ * a.ldk, a.ldk, (int)(a.dpad / K_TILE), lds, acc);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the spare tile request of the last step
    __syncthreads();                                    // every wave is done with both stages
    // dz = -g p here; the +g of the sampled token's column is added by a separate small kernel, so
    // the per-element work is one fma, one exp, one multiply and half a convert.  Rows past the last
    // token get g = 0; columns past V hold finite values that only ever meet zero weights.
    const Lane<S> L;
    char* region = lds + L.wave * (WJ * 32 * 256);   // WJ * 32 rows of 256 bytes per wave
    const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
    const int64_t jl_base = (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32);   // row in chunk
    const float zs = a.inv_temp * LOG2E;
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int row = jb * 32 + L.lj;
        const int64_t j = a.m0 + jl_base + row;
        const bool live = j < M;
        const float ngj = live ? -a.g[a.seqc[j]] * a.inv_temp : 0.f;
        const float nlse = live ? -a.lse_c[j] * LOG2E : 0.f;
        char* lrow = region + row * 256 + L.hi * 8;
        const int rx = row & 15;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float o[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    o[r] = ngj * __builtin_amdgcn_exp2f(fmaf(acc[ib][jb][q * 4 + r], zs, nlse));
                *(uint2*)(lrow + (((ib * 4 + q) ^ rx) * 16)) = pack_bf16x4(o[0], o[1], o[2], o[3]);
            }
    }
    // read back row-wise and store: lane l covers chunk l % 16 of row 4 t + l / 16
    const int c = L.lane & 15, r4 = L.lane >> 4;
    bf16_t* out = a.dz + (jl_base + r4) * a.ldz + i_base + c * 8;
#pragma unroll 8
    for (int tt = 0; tt < WJ * 8; ++tt) {
        const int row = tt * 4 + r4;
        const uint4 v = *(const uint4*)(region + row * 256 + ((c ^ (row & 15)) * 16));
        *(uint4*)(out + (int64_t)tt * 4 * a.ldz) = v;
    }
}

// ------------------------------------------------------------------------------------------ dh
template <class S>
__global__ __launch_bounds__(S::NT) void dh_kernel(DhArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesD = (int)(a.dpadR / S::BI);
    const TileId t = map_tile(blockIdx.x, tilesD, a.tilesM, a.gi > 0 ? a.gi : tilesD);
    if (!t.valid) return;
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.m0 + (int64_t)t.tj * S::BJ >= Mr) return;
    f32x16 acc[WI][WJ];
    mainloop<S>(a.Wdv + (int64_t)t.ti * S::BI * a.ldv, a.ldv,
                             a.dz + (int64_t)t.tj * S::BJ * a.ldv, a.ldv, (int)(a.Vpad / K_TILE), lds, acc);
    const Lane<S> L;
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
}

// ------------------------------------------------------------------------------------------ dw
template <class S>
__global__ __launch_bounds__(S::NT) void dw_kernel(DwArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesV = (int)(a.Vpad / S::BI), tilesD = (int)(a.dpadR / S::BJ);
    const TileId t = map_tile(blockIdx.x, tilesV, tilesD, a.gi);
    if (!t.valid) return;
    const int Mr = a.counts[CNT_MR];
    int64_t rows = (int64_t)Mr - a.m0;
    rows = rows < 0 ? 0 : (rows > a.Mc ? a.Mc : rows);
    if (rows == 0 && a.beta) return;   // nothing to add
    f32x16 acc[WI][WJ];
    mainloop_kmajor<S>(a.dz + (int64_t)t.ti * S::BI, a.ldz, a.Hc + (int64_t)t.tj * S::BJ, a.ldH,
                            (int)(rows / K_TILE), lds, acc);
    const Lane<S> L;
    const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
    const bool vec = (a.V % 4) == 0;
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
}

// Logit of the sampled token: zy[j] = inv_temp * <Hc[j, :], Wvd[tok_j, :]>, one wave per token row
// (16-byte loads, fp32 accumulation, fixed reduction tree).
__global__ __launch_bounds__(256) void token_logit_kernel(const bf16_t* __restrict__ Hc, const bf16_t* __restrict__ Wvd,
                                                          int64_t ldk, int64_t dpad, const int32_t* __restrict__ tokc,
                                                          const int32_t* __restrict__ counts, float inv_temp,
                                                          float* __restrict__ zy) {
    const int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= counts[CNT_M]) return;
    const int lane = threadIdx.x & 63;
    const bf16x8* h = (const bf16x8*)(Hc + j * ldk);
    const bf16x8* w = (const bf16x8*)(Wvd + (int64_t)tokc[j] * ldk);
    float acc = 0.f;
    for (int64_t c = lane; c < dpad / 8; c += 64) {
        const bf16x8 hv = h[c], wv = w[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf((float)hv[e], (float)wv[e], acc);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) zy[j] = acc * inv_temp;
}

// dz[row][tok_row] += g: the one-hot part of dz = g (onehot - p)
__global__ void token_onehot_kernel(bf16_t* __restrict__ dz, int64_t ldz, int64_t m0, int64_t rows,
                                    const int32_t* __restrict__ tokc, const int32_t* __restrict__ seqc,
                                    const float* __restrict__ g, float inv_temp, const int32_t* __restrict__ counts) {
    const int64_t jl = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t j = m0 + jl;
    if (jl >= rows || j >= counts[CNT_M]) return;
    bf16_t* p = dz + jl * ldz + tokc[j];
    const float cur = (float)__builtin_bit_cast(__bf16, *p);
    const __bf16 r = (__bf16)(cur + g[seqc[j]] * inv_temp);
    *p = __builtin_bit_cast(bf16_t, r);
}

template <class K>
void allow_lds(K kernel, int bytes) {
    (void)hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

int g_waves = 8;   // waves per workgroup: 4 (2 x 2 of 128 x 128) or 8 (2 x 4 of 128 x 64)

using G4 = Geo<2, 2, 4, 4>;        // 256 x 256, 4 waves
using G4_I128 = Geo<2, 2, 2, 4>;   // 128 x 256
using G4_J128 = Geo<2, 2, 4, 2>;   // 256 x 128
using G8 = Geo<2, 4, 4, 2>;        // 256 x 256, 8 waves
using G8_I128 = Geo<2, 4, 2, 2>;   // 128 x 256
using G8_J128 = Geo<2, 4, 4, 1>;   // 256 x 128
using G16 = Geo<2, 8, 4, 1>;       // 256 x 256, 16 waves of 128 x 32
using G16_I128 = Geo<2, 8, 2, 1>;  // 128 x 256
using G16_J128 = Geo<4, 4, 2, 1>;  // 256 x 128

template <class S>
void launch_fwd_lse_t(const FwdArgs& a, hipStream_t st) {
    allow_lds(fwd_lse_kernel<S>, S::LDS_BYTES);
    fwd_lse_kernel<S><<<grid_for(a.tilesV, a.tilesM), S::NT, S::LDS_BYTES, st>>>(a);
}
template <class S>
void launch_dz_t(const DzArgs& a, hipStream_t st) {
    allow_lds(dz_kernel<S>, S::LDS_BYTES);
    dz_kernel<S><<<grid_for(a.tilesV, a.tilesM), S::NT, S::LDS_BYTES, st>>>(a);
}
template <class S>
void launch_dh_t(const DhArgs& a, hipStream_t st) {
    allow_lds(dh_kernel<S>, S::LDS_BYTES);
    dh_kernel<S><<<grid_for((int)(a.dpadR / S::BI), a.tilesM), S::NT, S::LDS_BYTES, st>>>(a);
}
template <class S>
void launch_dw_t(const DwArgs& a, hipStream_t st) {
    allow_lds(dw_kernel<S>, S::LDS_BYTES);
    dw_kernel<S><<<grid_for((int)(a.Vpad / S::BI), (int)(a.dpadR / S::BJ)), S::NT, S::LDS_BYTES, st>>>(a);
}

}  // namespace

void set_waves_per_workgroup(int n) { g_waves = (n == 4 || n == 16) ? n : 8; }

void launch_fwd_lse(const FwdArgs& a, hipStream_t st) {
    if (g_waves == 16) launch_fwd_lse_t<G16>(a, st); else if (g_waves == 8) launch_fwd_lse_t<G8>(a, st); else launch_fwd_lse_t<G4>(a, st);
    const int64_t rows_max = (int64_t)a.tilesM * 256;
    token_logit_kernel<<<(unsigned)((rows_max + 3) / 4), 256, 0, st>>>(a.Hc, a.Wvd, a.ldk, a.dpad, a.tokc, a.counts,
                                                                     a.inv_temp, a.zy);
}
int fwd_slots_per_tile() { return 2; }

void launch_dz(const DzArgs& a, hipStream_t st) {
    if (g_waves == 16) launch_dz_t<G16>(a, st); else if (g_waves == 8) launch_dz_t<G8>(a, st); else launch_dz_t<G4>(a, st);
    const int64_t rows = (int64_t)a.tilesM * 256;
    token_onehot_kernel<<<(unsigned)((rows + 255) / 256), 256, 0, st>>>(a.dz, a.ldz, a.m0, rows, a.tokc, a.seqc, a.g,
                                                                      a.inv_temp, a.counts);
}

void launch_dh(const DhArgs& a, hipStream_t st) {
    if (a.dpadR % 256 == 0) {
        if (g_waves == 16) launch_dh_t<G16>(a, st); else if (g_waves == 8) launch_dh_t<G8>(a, st); else launch_dh_t<G4>(a, st);
    } else {   // d padded to a multiple of 128 only
        if (g_waves == 16) launch_dh_t<G16_I128>(a, st); else if (g_waves == 8) launch_dh_t<G8_I128>(a, st); else launch_dh_t<G4_I128>(a, st);
    }
}

void launch_dw(const DwArgs& a, hipStream_t st) {
    if (a.dpadR % 256 == 0) {
        if (g_waves == 16) launch_dw_t<G16>(a, st); else if (g_waves == 8) launch_dw_t<G8>(a, st); else launch_dw_t<G4>(a, st);
    } else {   // d padded to a multiple of 128 only
        if (g_waves == 16) launch_dw_t<G16_J128>(a, st); else if (g_waves == 8) launch_dw_t<G8_J128>(a, st); else launch_dw_t<G4_J128>(a, st);
    }
}

}  // namespace rapid
