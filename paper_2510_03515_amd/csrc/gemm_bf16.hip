// bf16 MFMA contractions of the hot path for gfx950 (CDNA4): one tiled main loop (two operand
// layouts) and four epilogues.
//   fwd_lse : logits tile  -> per-slot (max, sum exp) of the streaming log-softmax + gathered logit
//   dz      : logits tile  -> dz = g (onehot - softmax) / temperature, written as bf16
//   dh      : dH = dz . W^T          (contraction over the vocabulary)
//   dw      : dW (+)= H^T . dz       (contraction over the tokens of a row chunk)
//
// Tiling.  C[i][j] = sum_k A(i,k) B(j,k); operands are zero padded to whole tiles, so the loop has
// no bounds checks.  A workgroup of NWI x NWJ 64-lane waves owns a 256 x 256 tile (the largest whose
// fp32 accumulators a CU's registers hold, which minimises L2 -> LDS bytes per flop), each wave
// WI x WJ blocks of 32 x 32 computed with v_mfma_f32_32x32x16_bf16 (a lane feeds 8 consecutive k of
// one row).  The default is 2 x 4 waves of 128 x 64, two waves per SIMD.  K advances 64 elements
// per step through two LDS stages of 64 KiB (one barrier per step); operand tiles arrive by
// global_load_lds_dwordx4 (memory -> LDS without passing through registers; consecutive lanes fill
// consecutive 16-byte slots, so the LDS swizzle is applied to the global address).  The kernels
// are persistent: one workgroup per CU walks tile ids that are mapped to tiles so that the
// workgroups resident on an XCD (ids equal mod 8) own neighbouring tiles and share operand panels
// in that XCD's L2.
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
#include <atomic>
#include <utility>

#include "rapid_internal.h"

namespace rapid {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr float LOG2E = 1.4426950408889634f;

// Geometry of a workgroup: NWI x NWJ waves, each owning WI x WJ blocks of 32 x 32.
// 2 x 4 waves of 128 x 64 is the default (two waves per SIMD, which lets the hardware overlap one
// wave's LDS, barrier and memory-issue waits with the other's MFMAs at the price of 1.5x the LDS
// fragment reads); 2 x 2 waves of 128 x 128 (one wave per SIMD, 256 accumulator registers per lane)
// and 2 x 8 waves of 128 x 32 are selectable.
template <int NWI_, int NWJ_, int WI_, int WJ_>
struct Geo {
    static constexpr int NWI = NWI_, NWJ = NWJ_, WI = WI_, WJ = WJ_;
    static constexpr int NW = NWI * NWJ, NT = 64 * NW;
    static constexpr int BI = NWI * WI * 32, BJ = NWJ * WJ * 32;
    static constexpr int STAGE_BYTES = (BI + BJ) * 128;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

// Barrier without the memory fence of __syncthreads; the loops place their own waits before it.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

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

// LDS fragment reads and their waits are issued by hand.  With direct memory -> LDS loads in the
// loop the compiler's wait insertion falls back to lgkmcnt(0) before every MFMA block, which also
// waits for the reads just issued for the NEXT sub-step and so undoes the software pipelining.
// LDS reads of a wave complete in order, so "at most n reads outstanding" after issuing the next
// sub-step's n reads means exactly "the current sub-step's fragments have arrived".
__device__ __forceinline__ uint32_t lds_addr(const char* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}
template <int OFF>
__device__ __forceinline__ bf16x8 ds_read128(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
template <int OFF>
__device__ __forceinline__ s16x4 ds_read_tr64(uint32_t addr) {
    s16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
// waits until at most N LDS reads are outstanding, and makes the fragments depend on the wait
template <int N, int WI, int WJ>
__device__ __forceinline__ void wait_frags(Frags<WI, WJ>& f) {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N < 15 ? N : 15) : "memory");
#pragma unroll
    for (int ib = 0; ib < WI; ++ib) asm volatile("" : "+v"(f.a[ib]));
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) asm volatile("" : "+v"(f.b[jb]));
}

template <int WI, int WJ, int... IB, int... JB>
__device__ __forceinline__ void load_frags_seq(Frags<WI, WJ>& f, uint32_t a_addr, uint32_t b_addr,
                                               std::integer_sequence<int, IB...>, std::integer_sequence<int, JB...>) {
    ((f.a[IB] = ds_read128<IB * (32 * 128)>(a_addr)), ...);
    ((f.b[JB] = ds_read128<JB * (32 * 128)>(b_addr)), ...);
}
// a_addr / b_addr: LDS byte addresses of this lane's chunk in block 0 of each operand
template <int WI, int WJ>
__device__ __forceinline__ void load_frags(Frags<WI, WJ>& f, uint32_t a_addr, uint32_t b_addr) {
    load_frags_seq<WI, WJ>(f, a_addr, b_addr, std::make_integer_sequence<int, WI>{}, std::make_integer_sequence<int, WJ>{});
}

template <int WI, int WJ>
__device__ __forceinline__ void mma_block(const Frags<WI, WJ>& f, f32x16 (&acc)[WI][WJ]) {
#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
            acc[ib][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ib], f.b[jb], acc[ib][jb], 0, 0, 0);
}

// One MFMA block of a K step that also carries half of the step's tile-load requests (HALF = 0 / 1),
// one request after every few MFMAs.  A memory instruction holds its wave at issue until the memory
// pipeline accepts it, and that pipeline takes most of a step to accept a whole stage; requests
// bunched at the top of the step kept every wave out of its MFMAs for hundreds of cycles, spread out
// they are accepted at once and the SIMD's other wave fills the gaps.
// A wave makes T requests per step, numbered in the order `request(r)` is to be called; the block with
// HALF = 0 carries the first half of them, request_first_half makes the same ones without MFMAs.
template <class S, int HALF, int T, class F>
__device__ __forceinline__ void mma_block_requesting(const Frags<S::WI, S::WJ>& f, f32x16 (&acc)[S::WI][S::WJ],
                                                     F&& request) {
    constexpr int NB = S::WI * S::WJ;
#pragma unroll
    for (int ib = 0; ib < S::WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < S::WJ; ++jb) {
            acc[ib][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ib], f.b[jb], acc[ib][jb], 0, 0, 0);
            const int slot = HALF * NB + ib * S::WJ + jb;
#pragma unroll
            for (int r = 0; r < T; ++r)
                if (r * 2 * NB / T == slot) {
                    __builtin_amdgcn_sched_barrier(0);
                    request(r);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
}
template <class S, int T, class F>
__device__ __forceinline__ void request_first_half(F&& request) {
    constexpr int NB = S::WI * S::WJ;
#pragma unroll
    for (int r = 0; r < T; ++r)
        if (r * 2 * NB / T < NB) request(r);
}
__device__ __forceinline__ void load_to_lds_16(const char* gp, char* lp) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                     (__attribute__((address_space(3))) void*)lp, 16, 0, 0);
}

// Scheduling fence: nothing is moved across it.  The K step is written in the order that software-
// pipelines it (fragments of the next sub-step are requested before the MFMAs of the current one,
// tile requests sit between given MFMAs) and the fences keep that order.
__device__ __forceinline__ void fence() { __builtin_amdgcn_sched_barrier(0); }

struct NoPace {
    __device__ __forceinline__ void operator()(int) const {}
};

// Keeps all workgroups of a launch within a few K steps of each other, so that a W panel one XCD
// has pulled through the memory-side cache is still there when the others ask for it.  Every
// `every` K steps thread 0 counts its workgroup in and polls, a bounded number of times, until the
// others of the round have arrived; the rest of the workgroup meets it at the next barrier.  Purely
// a pacing hint: nothing depends on it, a poll that runs out sets the counter's top bit, which
// satisfies every later target, and the kernel goes on unpaced.
struct GridPace {
    unsigned* ctr;      // arrival counter, zero at launch
    unsigned base;      // arrivals of the rounds before this tile
    unsigned n;         // workgroups that work on a tile in this round
    int every;          // K steps between meetings (power of two), 0 = off
    __device__ __forceinline__ void operator()(int kt) const {
        if (every == 0 || ((kt + 1) & (every - 1)) != 0) return;
        if (threadIdx.x == 0) {
            const unsigned target = base + n * (unsigned)((kt + 1) / every);
            __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int polls = 0;
            while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (++polls == 256) {
                    __hip_atomic_fetch_or(ctr, 0x80000000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
        }
    }
};

// acc += A_tile . B_tile^T over `ktiles` steps of 64.  A / B point at the tile's first row, k = 0.
template <class S, class Pace = NoPace>
__device__ __forceinline__ void mainloop(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                                         int64_t ldb, int ktiles, char* lds, f32x16 (&acc)[S::WI][S::WJ],
                                         int step_a = 128, int step_b = 128, Pace pace = Pace()) {
    constexpr int WI = S::WI, WJ = S::WJ;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_i = wave % S::NWI, wave_j = wave / S::NWI;

    // global side of the tile loads: lane l of a wave covers row l/8 of the wave's 8-row band and
    // the chunk that belongs at slot l%8 of that row; a wave's bands are 8 * (waves that share the
    // tile) rows apart.
    const int gchunk = (lane & 7) ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);
    const uint32_t voff_a = (uint32_t)(((int64_t)(lane >> 3) * lda + gchunk * 8) * 2);
    const uint32_t voff_b = (uint32_t)(((int64_t)(lane >> 3) * ldb + gchunk * 8) * 2);
    const char* ga = (const char*)(A + (int64_t)(wave * 8) * lda);
    const char* gb = (const char*)(B + (int64_t)(wave * 8) * ldb);
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

    // A workgroup runs tile after tile: everybody must be done with the LDS stages of the tile before
    // (its last reads, its trailing requests, a staged epilogue) before they are filled again.
    lds_barrier();
    issue_tile_load<S::BI, S::NW>(ga, voff_a, (int64_t)(8 * S::NW) * lda * 2, lds + lds_wave_off);
    issue_tile_load<S::BJ, S::NW>(gb, voff_b, (int64_t)(8 * S::NW) * ldb * 2, lds + S::BI * 128 + lds_wave_off);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();

    // One K step on stage `cur` = kt % 2 (its first fragments f0 were read at the end of the step before,
    // and the first half of tile kt+1 was requested there too):
    //   read f1 (sub-step 1) | MFMA f0 + second half of the requests for tile kt+1
    //   read f0 (sub-step 2) | MFMA f1
    //   read f1 (sub-step 3) | MFMA f0
    //   wait: own requests landed, own reads of `cur` done; barrier
    //   read f0 of tile kt+1 | MFMA f1 + first half of the requests for tile kt+2 (into `cur`)
    // After the barrier tile kt+1 is complete and nobody reads `cur` any more.  Steps past the last
    // tile re-request the last tile into the idle stage, which keeps the loop free of branches and
    // every address in bounds.  (Skipping those requests with a uniform branch each was tried: the logits
    // kernels, where they are 6 % of the memory -> LDS traffic, got 2 % slower and dHidden 5 %.)
    Frags<WI, WJ> f0, f1;
    constexpr int NR = WI + WJ;   // LDS reads per sub-step
    constexpr int RA = S::BI / (8 * S::NW), RB = S::BJ / (8 * S::NW), SR = 8 * S::NW;
    char* dst = lds + S::STAGE_BYTES;   // stage the requests go to
    auto request = [&](int r) {
        if (r < RA)
            load_to_lds_16(ga + (int64_t)(r * SR) * lda * 2 + voff_a, dst + lds_wave_off + r * (SR * 128));
        else
            load_to_lds_16(gb + (int64_t)((r - RA) * SR) * ldb * 2 + voff_b,
                           dst + S::BI * 128 + lds_wave_off + (r - RA) * (SR * 128));
    };
    {
        const uint32_t la = lds_addr(lds) + a_off, lb = lds_addr(lds) + b_off;
        load_frags<WI, WJ>(f0, la + xo[0], lb + xo[0]);
        ga += ktiles > 1 ? step_a : 0;
        gb += ktiles > 1 ? step_b : 0;
        request_first_half<S, RA + RB>(request);   // of tile 1
        // A register that an LDS read (issued from inline assembly) is still writing must not meet
        // a compiler-made copy, and copies appear where control flow splits or joins: every read is
        // therefore waited for in the block that issued it.
        wait_frags<0>(f0);
    }
    for (int kt = 0; kt < ktiles; ++kt) {
        char* cur = lds + (kt & 1) * S::STAGE_BYTES;
        char* nxt = lds + ((kt + 1) & 1) * S::STAGE_BYTES;
        const uint32_t la = lds_addr(cur) + a_off, lb = lds_addr(cur) + b_off;
        const uint32_t na = lds_addr(nxt) + a_off, nb = lds_addr(nxt) + b_off;
        fence();
        load_frags<WI, WJ>(f1, la + xo[1], lb + xo[1]);
        fence();
        dst = nxt;
        mma_block_requesting<S, 1, RA + RB>(f0, acc, request);
        fence();
        load_frags<WI, WJ>(f0, la + xo[2], lb + xo[2]);
        wait_frags<NR>(f1);
        fence();
        mma_block<WI, WJ>(f1, acc);
        fence();
        load_frags<WI, WJ>(f1, la + xo[3], lb + xo[3]);
        wait_frags<NR>(f0);
        fence();
        mma_block<WI, WJ>(f0, acc);
        fence();
        wait_frags<0>(f1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        pace(kt);   // no LDS read or tile request is in flight here
        load_frags<WI, WJ>(f0, na + xo[0], nb + xo[0]);
        fence();
        ga += (kt + 2 < ktiles) ? step_a : 0;
        gb += (kt + 2 < ktiles) ? step_b : 0;
        dst = cur;
        mma_block_requesting<S, 0, RA + RB>(f1, acc, request);
        fence();
        wait_frags<0>(f0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests for steps that do not exist
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
template <int COLS, int NW, int STEP = 64>         // STEP: rows (contraction indices) per K step
struct KMajor {
    static constexpr int ROW_BYTES = COLS * 2;
    static constexpr int CPR = COLS / 8;          // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;          // rows covered by one wave-wide load instruction
    static constexpr int ROUNDS = STEP / (NW * RPI);
    static constexpr int ROUND_ROWS = NW * RPI;
    static constexpr int SEGS = CPR / 4;          // 64-byte segments per row
    static constexpr int TILE_BYTES = STEP * ROW_BYTES;
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

template <int OFF>
__device__ __forceinline__ bf16x8 read_tr_frag(uint32_t a0, uint32_t a1) {
    const s16x4 lo = ds_read_tr64<OFF>(a0);
    const s16x4 hi = ds_read_tr64<OFF>(a1);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// xa / xb: this lane's LDS byte offsets (two half-fragments per block) within a stage, sub-step 0
template <int KS, class S>
__device__ __forceinline__ void load_frags_kmajor(Frags<S::WI, S::WJ>& f, uint32_t cur, const int (&xa)[S::WI][2],
                                                  const int (&xb)[S::WJ][2]) {
    constexpr int OA = KS * 16 * KMajor<S::BI, S::NW>::ROW_BYTES, OB = KS * 16 * KMajor<S::BJ, S::NW>::ROW_BYTES;
#pragma unroll
    for (int ib = 0; ib < S::WI; ++ib) f.a[ib] = read_tr_frag<OA>(cur + xa[ib][0], cur + xa[ib][1]);
#pragma unroll
    for (int jb = 0; jb < S::WJ; ++jb) f.b[jb] = read_tr_frag<OB>(cur + xb[jb][0], cur + xb[jb][1]);
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

    int xa[WI][2], xb[WJ][2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
#pragma unroll
        for (int ib = 0; ib < WI; ++ib) xa[ib][r] = base_a[r] ^ (ib * 64);
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) xb[jb][r] = base_b[r] ^ (jb * 64);
    }
    constexpr int NR = 2 * (WI + WJ);   // LDS reads per sub-step

#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.f;

    if (ktiles <= 0) return;

    lds_barrier();   // see mainloop
    issue_kmajor_load<S::BI, S::NW>(ga, voff_a, round_a, lds + lds_wave_a);
    issue_kmajor_load<S::BJ, S::NW>(gb, voff_b, round_b, lds + lds_wave_b);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();

    // same step structure as mainloop
    Frags<WI, WJ> f0, f1;
    char* dst = lds + S::STAGE_BYTES;
    auto request = [&](int r) {
        if (r < KA::ROUNDS)
            load_to_lds_16(ga + r * round_a + voff_a, dst + lds_wave_a + r * (KA::ROUND_ROWS * KA::ROW_BYTES));
        else
            load_to_lds_16(gb + (r - KA::ROUNDS) * round_b + voff_b,
                           dst + lds_wave_b + (r - KA::ROUNDS) * (KB::ROUND_ROWS * KB::ROW_BYTES));
    };
    constexpr int T = KA::ROUNDS + KB::ROUNDS;
    {
        load_frags_kmajor<0, S>(f0, lds_addr(lds), xa, xb);
        const bool more = ktiles > 1;
        ga += more ? step_a : 0;
        gb += more ? step_b : 0;
        request_first_half<S, T>(request);   // of tile 1
        wait_frags<0>(f0);
    }
    for (int kt = 0; kt < ktiles; ++kt) {
        char* cur = lds + (kt & 1) * S::STAGE_BYTES;
        char* nxt = lds + ((kt + 1) & 1) * S::STAGE_BYTES;
        const uint32_t lc = lds_addr(cur), ln = lds_addr(nxt);
        fence();
        load_frags_kmajor<1, S>(f1, lc, xa, xb);
        fence();
        dst = nxt;
        mma_block_requesting<S, 1, T>(f0, acc, request);
        fence();
        load_frags_kmajor<2, S>(f0, lc, xa, xb);
        wait_frags<NR>(f1);
        fence();
        mma_block<WI, WJ>(f1, acc);
        fence();
        load_frags_kmajor<3, S>(f1, lc, xa, xb);
        wait_frags<NR>(f0);
        fence();
        mma_block<WI, WJ>(f0, acc);
        fence();
        wait_frags<0>(f1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        load_frags_kmajor<0, S>(f0, ln, xa, xb);
        fence();
        const bool more = kt + 2 < ktiles;
        ga += more ? step_a : 0;
        gb += more ? step_b : 0;
        dst = cur;
        mma_block_requesting<S, 0, T>(f1, acc, request);
        fence();
        wait_frags<0>(f0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests for steps that do not exist
}

// The same contraction with K steps of 32 rows through NST LDS stages (NST x 32 rows = the same LDS as two
// steps of 64), the requests NST - 1 steps ahead of the MFMAs: the streamed operand of dW comes from HBM, and
// one step of lead is less than a trip there.  Same LDS layout per row, same fragments, same order of
// summation per accumulator: identical results.
template <class S, int NST>
__device__ __forceinline__ void mainloop_kmajor32(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                                                  int64_t ldb, int ksteps, char* lds, f32x16 (&acc)[S::WI][S::WJ]) {
    constexpr int WI = S::WI, WJ = S::WJ;
    using KA = KMajor<S::BI, S::NW, 32>;
    using KB = KMajor<S::BJ, S::NW, 32>;
    static_assert(KA::ROUNDS >= 1 && KB::ROUNDS >= 1, "a wave instruction must not span more than a step");
    constexpr int STAGE = KA::TILE_BYTES + KB::TILE_BYTES, D = NST - 1, T = KA::ROUNDS + KB::ROUNDS;
    static_assert(NST * STAGE <= S::LDS_BYTES, "stages must fit the kernel's LDS");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_i = wave % S::NWI, wave_j = wave / S::NWI;

    auto lane_voff = [&](int cpr, int segs, int rpi, int64_t ld) -> uint32_t {
        const int lrow = lane / cpr, p = lane % cpr;
        const int row_low = (wave * rpi + lrow) & (segs - 1);
        const int gseg = (p >> 2) ^ row_low;
        return (uint32_t)(((int64_t)lrow * ld + (gseg * 4 + (p & 3)) * 8) * 2);
    };
    const uint32_t voff_a = lane_voff(KA::CPR, KA::SEGS, KA::RPI, lda);
    const uint32_t voff_b = lane_voff(KB::CPR, KB::SEGS, KB::RPI, ldb);
    const char* ga = (const char*)(A + (int64_t)(wave * KA::RPI) * lda) + voff_a;
    const char* gb = (const char*)(B + (int64_t)(wave * KB::RPI) * ldb) + voff_b;
    const int64_t round_a = (int64_t)KA::ROUND_ROWS * lda * 2, round_b = (int64_t)KB::ROUND_ROWS * ldb * 2;
    const int64_t step_a = 32 * lda * 2, step_b = 32 * ldb * 2;
    const int lds_wave_a = wave * KA::RPI * KA::ROW_BYTES;
    const int lds_wave_b = KA::TILE_BYTES + wave * KB::RPI * KB::ROW_BYTES;

    const int q = (lane & 15) >> 2;
    const int sub_bytes = (2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 16 + 8 * (lane & 1);
    const int rowpart = 8 * (lane >> 5) + q;
    int xa[WI][2], xb[WJ][2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int sw = 4 * r + q;   // low bits of the row this lane addresses in half r
        const int base_a = (rowpart + 4 * r) * KA::ROW_BYTES + ((((wave_i * WI) ^ (sw & (KA::SEGS - 1))) * 64)) + sub_bytes;
        const int base_b = KA::TILE_BYTES + (rowpart + 4 * r) * KB::ROW_BYTES +
                           ((((wave_j * WJ) ^ (sw & (KB::SEGS - 1))) * 64)) + sub_bytes;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib) xa[ib][r] = base_a ^ (ib * 64);
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) xb[jb][r] = base_b ^ (jb * 64);
    }

#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.f;
    if (ksteps <= 0) return;

    int src_step = 0;       // K step the next requests fetch (clamped to the last one), and the stage they go to
    char* dst;
    auto request = [&](int r) {
        if (r < KA::ROUNDS)
            load_to_lds_16(ga + src_step * step_a + r * round_a, dst + lds_wave_a + r * (KA::ROUND_ROWS * KA::ROW_BYTES));
        else
            load_to_lds_16(gb + src_step * step_b + (r - KA::ROUNDS) * round_b,
                           dst + lds_wave_b + (r - KA::ROUNDS) * (KB::ROUND_ROWS * KB::ROW_BYTES));
    };
    lds_barrier();   // see mainloop
#pragma unroll
    for (int st = 0; st < D; ++st) {
        dst = lds + st * STAGE;
        src_step = st < ksteps ? st : ksteps - 1;
#pragma unroll
        for (int r = 0; r < T; ++r) request(r);
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * T) : "memory");   // step 0 has landed
    lds_barrier();
    Frags<WI, WJ> f0, f1;
    load_frags_kmajor<0, S>(f0, lds_addr(lds), xa, xb);
    wait_frags<0>(f0);
    int cur_i = 0, fil_i = D;
    for (int kt = 0; kt < ksteps; ++kt) {
        const uint32_t lc = lds_addr(lds + cur_i * STAGE);
        const int nxt_i = cur_i + 1 == NST ? 0 : cur_i + 1;
        const uint32_t ln = lds_addr(lds + nxt_i * STAGE);
        fence();
        load_frags_kmajor<1, S>(f1, lc, xa, xb);
        fence();
        dst = lds + fil_i * STAGE;
        src_step = kt + D < ksteps ? kt + D : ksteps - 1;
        mma_block_requesting<S, 0, 2 * T>(f0, acc, request);   // the T requests for step kt + D, spread over the MFMAs
        fence();
        wait_frags<0>(f1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * T) : "memory");   // own requests for step kt + 1 have landed
        lds_barrier();
        load_frags_kmajor<0, S>(f0, ln, xa, xb);
        fence();
        mma_block<WI, WJ>(f1, acc);
        fence();
        wait_frags<0>(f0);
        cur_i = nxt_i;
        fil_i = fil_i + 1 == NST ? 0 : fil_i + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests for steps that do not exist
}

// Workgroup id -> tile.  Hardware deals consecutive workgroup ids round-robin to the 8 XCDs (each
// with its own L2), so id % 8 picks the XCD and id / 8 the position in that XCD's contiguous share
// of a grouped order: GI tiles along i for one j, then the next j, ... so that workgroups resident
// together on an XCD re-use each other's operand panels out of L2.
struct TileId { int ti, tj; bool valid; };
// position `vid` of the grouped order -> tile
__device__ __forceinline__ TileId tile_of_vid(int vid, int tilesI, int tilesJ, int GI) {
    const int total = tilesI * tilesJ;
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
__device__ __forceinline__ TileId map_tile(int pid, int tilesI, int tilesJ, int GI) {
    const int per = (tilesI * tilesJ + 7) / 8;
    return tile_of_vid((pid & 7) * per + (pid >> 3), tilesI, tilesJ, GI);
}

__host__ __device__ inline int ids_for(int tilesI, int tilesJ) { return (int)(((int64_t)tilesI * tilesJ + 7) / 8 * 8); }
// The kernels are persistent: one workgroup per CU (LDS admits no more) walks the ids
// blockIdx.x, blockIdx.x + gridDim.x, ...; gridDim.x is a multiple of 8, so a workgroup stays on its
// XCD's share of the order and the workgroups of an XCD stay on neighbouring tiles.  This saves the
// launch gap between workgroups and the dispatch of the ids whose tiles hold no token rows.
std::atomic<int> g_num_cu{256};
inline unsigned grid_for(int tilesI, int tilesJ) {
    const int ids = ids_for(tilesI, tilesJ), cus = g_num_cu.load() / 8 * 8;
    return (unsigned)(ids < cus ? ids : cus);
}

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

// A 256 x 256 tile of bf16 values leaves through LDS so that it reaches memory as whole 256-byte row
// segments.  Each wave owns a private region (its WJ * 32 token rows x 128 columns, 256 bytes per
// row; the regions are exactly the two idle LDS stages).  A lane writes its runs of 4 consecutive
// columns (8 bytes) at 16-byte chunk c ^ (row % 16) of the row, then the wave reads the region back
// row-wise, 16 lanes x 16 bytes per row, and stores 4 full rows per instruction.  The stores are
// streamed (non-temporal): the destination is far larger than the L2s and must not push the
// operand panels out.  `value(ib, jb, v)` is the element the lane holds in accumulator register v of
// block (ib, jb); `out` points at (first row of the wave, first column of the wave) of the tile.
// All waves must be done with both LDS stages (barrier) before the call.
template <class S, class F>
__device__ __forceinline__ void store_tile_through_lds(char* lds, const Lane<S>& L, bf16_t* out, int64_t ld, F&& value) {
    constexpr int WI = S::WI, WJ = S::WJ;
    static_assert(WI == 4, "laid out for 128 columns (256 bytes) per wave row");
    char* region = lds + L.wave * (WJ * 32 * 256);
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int row = jb * 32 + L.lj;
        char* lrow = region + row * 256 + L.hi * 8;
        const int rx = row & 15;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(uint2*)(lrow + (((ib * 4 + q) ^ rx) * 16)) =
                    pack_bf16x4(value(ib, jb, q * 4), value(ib, jb, q * 4 + 1), value(ib, jb, q * 4 + 2),
                                value(ib, jb, q * 4 + 3));
    }
    // read back row-wise and store: lane l covers chunk l % 16 of row 4 t + l / 16
    const int c = L.lane & 15, r4 = L.lane >> 4;
    bf16_t* o = out + (int64_t)r4 * ld + c * 8;
#pragma unroll 8
    for (int tt = 0; tt < WJ * 8; ++tt) {
        const int row = tt * 4 + r4;
        const uint4 v = *(const uint4*)(region + row * 256 + ((c ^ (row & 15)) * 16));
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4*)(o + (int64_t)tt * 4 * ld));
    }
}

// ------------------------------------------------------------------------------------- fwd_lse
// STORE: also keep, for a backward that reloads them instead of recomputing the logits, the tile's
// scaled probabilities u[j][v] = exp(z[j][v] - r[j]) in bf16 in a.zc.  The reference r[j] (a.refz) is
// known before the sweep, so the row's log-sum-exp is not needed to write u, and the backward needs
// one factor per row, -g exp(r - lse), instead of a pass over the stored tile.  r is the logit of
// the row's sampled token minus its behaviour log-prob: the behaviour policy's log-sum-exp, moved by
// the token's own drift, so u is close to the probability itself; without behaviour log-probs it is
// the sampled token's logit and u = p_v / p_y.  The exponent is clamped at 2^115 (a logit 79 above
// the reference); a clamp sets RAPID_STATUS_LOGIT_RANGE.
//
// Epilogue of a logits tile: per token row j (one lane pair) the max and the sum of exponentials over this
// wave's 128 vocabulary columns.  The logit of the sampled token is gathered by a separate small kernel,
// so the per-element work is one max, one fma, one exp and one add (STORE: and one multiply).
template <class S, bool STORE>
__device__ __forceinline__ void fwd_epilogue(const FwdArgs& a, const TileId& t, int64_t j_tile, int M, char* lds,
                                             f32x16 (&acc)[S::WI][S::WJ]) {
    constexpr int WI = S::WI, WJ = S::WJ;
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
    float m[WJ], nm[WJ], l[WJ];
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        float mx = -INFINITY;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[ib][jb][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        m[jb] = mx;
        nm[jb] = (mx == -INFINITY) ? 0.f : -mx * zs;
        l[jb] = 0.f;
    }
    if (STORE) {
        float f[WJ];   // exp(wave maximum - reference): turns exp(z - maximum) into exp(z - reference)
        bool clamped = false;
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb) {
            const int64_t j = j_tile + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
            const float r2 = j < M ? a.refz[j] * LOG2E : 0.f;   // rows past the last token: zero logits
            float e2 = m[jb] * zs - r2;                        // -inf for a wave of padding columns only
            if (e2 > 115.f) { e2 = 115.f; clamped = true; }
            f[jb] = __builtin_amdgcn_exp2f(e2);
        }
        if (clamped && a.dev_status) atomicOr(a.dev_status, RAPID_STATUS_LOGIT_RANGE);
        __syncthreads();   // every wave is done with both stages
        store_tile_through_lds<S>(lds, L,
                                  a.zc + (j_tile - a.zc_row0 + L.wave_j * (WJ * 32)) * a.ldz + (int64_t)t.ti * S::BI + L.wave_i * (WI * 32),
                                  a.ldz, [&](int ib, int jb, int v) {
                                      const float e = __builtin_amdgcn_exp2f(fmaf(acc[ib][jb][v], zs, nm[jb]));
                                      l[jb] += e;
                                      return e * f[jb];
                                  });
    } else {
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int ib = 0; ib < WI; ++ib)
#pragma unroll
                for (int v = 0; v < 16; ++v) l[jb] += __builtin_amdgcn_exp2f(fmaf(acc[ib][jb][v], zs, nm[jb]));
    }
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int64_t j = j_tile + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
        const float ls = l[jb] + __shfl_xor(l[jb], 32, 64);
        if (L.hi == 0) {
            a.part_max[slot * a.ld_part + (j - a.part_row0)] = m[jb] * a.inv_temp;
            a.part_sum[slot * a.ld_part + (j - a.part_row0)] = ls;
        }
    }
}

// one workgroup per CU on 256 x 256 tiles: the logits tile on MFMA, then the epilogue above
template <class S, bool STORE>
__global__ __launch_bounds__(S::NT) void fwd_lse_kernel(FwdArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.row0 >= Mr) return;
    // the order (and with it the split over the XCDs) covers the row tiles that hold tokens only
    const int tilesM = min(a.tilesM, (int)((Mr - a.row0 + S::BJ - 1) / S::BJ));
    for (int pid = blockIdx.x, ids = ids_for(a.tilesV, tilesM); pid < ids; pid += gridDim.x) {
    const TileId t = map_tile(pid, a.tilesV, tilesM, a.gi);
    const int64_t j_tile = a.row0 + (int64_t)t.tj * S::BJ;   // first token row of the tile
    if (!t.valid) continue;
    f32x16 acc[WI][WJ];
    mainloop<S>(a.Wvd + (int64_t)t.ti * S::BI * a.ldk, a.ldk, a.Hc + j_tile * a.ldk, a.ldk, (int)(a.dpad / K_TILE), lds,
                acc);
    fwd_epilogue<S, STORE>(a, t, j_tile, M, lds, acc);
    }
}

// ---------------------------------------------------------------- fwd_lse, two workgroups per CU
// The tiles of the logits kernels are short (K = d is a few dozen steps) and end in an epilogue the MFMA
// pipe does not take part in (max, exp, sum over the accumulators; STORE: the staged store).  With one
// workgroup per CU nothing else is resident to use the pipe meanwhile.  This variant runs TWO workgroups
// of 4 waves per CU, each on a 256 (vocabulary) x 128 (token rows) tile, so one workgroup's epilogue and
// tile fill overlap the other's main loop.  Each wave still owns 128 x 64 (the same fragments per MFMA as
// the 8-wave kernel).  For two workgroups to fit, K advances 32 per step through three LDS stages of
// 24 KiB (72 KiB per workgroup).  Half-line rows would double the L2 requests, so W comes from a copy that
// is blocked per (256-row tile, K step): 16 KiB contiguous, already in the LDS order, and a request is a
// straight 1 KiB copy; the hidden rows stay row-major (half a line per row and step, a third of the bytes).
//
// LDS layout of a stage: 256 W rows, then 128 hidden rows, 64 bytes each = 4 chunks of 16 bytes; chunk c of
// row r sits at position c ^ ((r >> 2) & 3), which makes the ds_read_b128 fragment reads conflict free
// (16 consecutive lanes = 16 consecutive rows of one chunk index cover 256 distinct bytes).
template <int NWJ_, int NSTAGE_, int WJ_ = 2>
struct FwdK32 {
    using S = Geo<2, NWJ_, 4, WJ_>;                // 2 x NWJ waves of 128 x (32 WJ): a 256 x (32 WJ NWJ) tile
    static constexpr int K_STEP = 32, NSTAGE = NSTAGE_, NW = 2 * NWJ_;
    static constexpr int A_BYTES = 256 * 64, B_BYTES = S::BJ * 64, STAGE = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = STAGE * NSTAGE;
    static constexpr int RA = 16 / NW, RB = S::BJ / 16 / NW, R = RA + RB;   // 1 KiB requests per wave and step
};
using Fwd2 = FwdK32<2, 3>;   // two workgroups per CU: 4 waves, 256 x 128, 72 KiB
using Fwd3 = FwdK32<4, 4>;   // one workgroup per CU: 8 waves, 256 x 256, 128 KiB, requests three steps ahead
using Fwd4 = FwdK32<2, 4, 4>;   // the same with 4 waves of 128 x 128 (a third fewer LDS fragment reads per MFMA)

// acc = W_tile . H_tile^T over `ksteps` steps of 32.  wblk: the tile's first block of the blocked copy of W
// (ksteps blocks of 16 KiB follow each other); B: first hidden row of the tile, row-major, ldb elements.
// The requests run NSTAGE - 1 steps ahead of the MFMAs.
template <class F2>
__device__ __forceinline__ void mainloop32(const char* __restrict__ wblk, const bf16_t* __restrict__ B, int64_t ldb,
                                           int ksteps, char* lds, f32x16 (&acc)[4][F2::S::WJ]) {
    using S = typename F2::S;
    constexpr int WI = 4, WJ = S::WJ, NW = F2::NW, RA = F2::RA, R = F2::R, NST = F2::NSTAGE, D = NST - 1;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_i = wave & 1, wave_j = wave >> 1;

    // requests: 1 KiB each; request r of a wave is unit r NW + wave of its operand (W: linear; hidden rows: 16 rows)
    const char* ga = wblk + wave * 1024 + lane * 16;
    const int gchunk = (lane & 3) ^ ((lane >> 4) & 3);            // chunk that belongs at slot lane % 4 of row lane / 4
    const char* gb = (const char*)(B + (int64_t)(wave * 16 + (lane >> 2)) * ldb + gchunk * 8);
    const int64_t b_round = (int64_t)(16 * NW) * ldb * 2;         // the wave's next 16 rows
    const int dst_wave = wave * 1024;

    // fragment reads
    const int frow = lane & 31, fhi = lane >> 5;
    const int x0 = (fhi ^ ((frow >> 2) & 3)) * 16, x1 = x0 ^ 32;  // chunk 2 ks + fhi at its swizzled position
    const int a_off = (wave_i * 128 + frow) * 64;
    const int b_off = F2::A_BYTES + (wave_j * (WJ * 32) + frow) * 64;

#pragma unroll
    for (int ib = 0; ib < WI; ++ib)
#pragma unroll
        for (int jb = 0; jb < WJ; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.f;
    if (ksteps <= 0) return;

    int src_step = 0;       // K step the next requests fetch (clamped to the last one: the loop has no branches
    char* dst;              // and every address stays in bounds), and the stage they go to
    auto request = [&](int r) {
        if (r < RA)
            load_to_lds_16(ga + (int64_t)src_step * F2::A_BYTES + r * (NW * 1024), dst + dst_wave + r * (NW * 1024));
        else
            load_to_lds_16(gb + (int64_t)src_step * 64 + (r - RA) * b_round,
                           dst + F2::A_BYTES + dst_wave + (r - RA) * (NW * 1024));
    };
    auto read_frags = [&](Frags<WI, WJ>& f, const char* stage, int x) {
        const uint32_t la = lds_addr(stage) + a_off + x, lb = lds_addr(stage) + b_off + x;
        f.a[0] = ds_read128<0>(la); f.a[1] = ds_read128<2048>(la); f.a[2] = ds_read128<4096>(la); f.a[3] = ds_read128<6144>(la);
        f.b[0] = ds_read128<0>(lb); f.b[1] = ds_read128<2048>(lb);
        if constexpr (WJ == 4) { f.b[2] = ds_read128<4096>(lb); f.b[3] = ds_read128<6144>(lb); }
    };

    // everybody is done with the stages of the tile before (reads, trailing requests, a staged epilogue)
    lds_barrier();
#pragma unroll
    for (int st = 0; st < D; ++st) {                  // steps 0 .. D-1 into stages 0 .. D-1
        dst = lds + st * F2::STAGE;
        src_step = st < ksteps ? st : ksteps - 1;
#pragma unroll
        for (int r = 0; r < R; ++r) request(r);
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * R) : "memory");   // step 0 has landed (loads complete in order)
    lds_barrier();
    Frags<WI, WJ> f0, f1;
    read_frags(f0, lds, x0);
    wait_frags<0>(f0);
    // One K step on stage `cur` (its first fragments f0 are in registers):
    //   read f1 (second half of the step) | MFMA f0 + the requests for step kt+D into stage (kt+D) % NSTAGE
    //   wait: own reads of `cur` done, own requests for step kt+1 landed; barrier
    //   read f0 of step kt+1              | MFMA f1
    // The stage the requests go to was read during step kt-1, and everybody passed the barrier at the end of it.
    int cur_i = 0, fil_i = D;
    for (int kt = 0; kt < ksteps; ++kt) {
        char* cur = lds + cur_i * F2::STAGE;
        const int nxt_i = cur_i + 1 == NST ? 0 : cur_i + 1;
        char* nxt = lds + nxt_i * F2::STAGE;
        fence();
        read_frags(f1, cur, x1);
        fence();
        dst = lds + fil_i * F2::STAGE;
        src_step = kt + D < ksteps ? kt + D : ksteps - 1;
        mma_block_requesting<S, 0, 2 * R>(f0, acc, request);   // the R requests spread over the 8 MFMAs
        fence();
        wait_frags<0>(f1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * R) : "memory");
        lds_barrier();
        read_frags(f0, nxt, x0);
        fence();
        mma_block<WI, WJ>(f1, acc);
        fence();
        wait_frags<0>(f0);
        cur_i = nxt_i;
        fil_i = fil_i + 1 == NST ? 0 : fil_i + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests for steps that do not exist
}

template <class F2, bool STORE>
__global__ __launch_bounds__(64 * F2::NW, (F2::NW == 4 && F2::S::WJ == 2) ? 2 : 1) void fwd_lse2_kernel(FwdArgs a) {
    using S = typename F2::S;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.row0 >= Mr) return;
    // the order covers the row tiles that hold tokens only
    const int tilesM = min(a.tilesM * (256 / S::BJ), (int)((Mr - a.row0 + S::BJ - 1) / S::BJ));
    const int ksteps = (int)(a.dpad / F2::K_STEP);
    for (int pid = blockIdx.x, ids = ids_for(a.tilesV, tilesM); pid < ids; pid += gridDim.x) {
        const TileId t = map_tile(pid, a.tilesV, tilesM, a.gi);
        if (!t.valid) continue;
        const int64_t j_tile = a.row0 + (int64_t)t.tj * S::BJ;
        f32x16 acc[4][S::WJ];
        mainloop32<F2>((const char*)a.WvdB + (int64_t)t.ti * ksteps * F2::A_BYTES, a.Hc + j_tile * a.ldk, a.ldk, ksteps, lds, acc);
        fwd_epilogue<S, STORE>(a, t, j_tile, M, lds, acc);
    }
}

// W as the two-workgroup forward reads it: for every 256-row tile and K step of 32 a 16 KiB block, row r's
// chunk c (8 elements) at position c ^ ((r >> 2) & 3) of the row's 64 bytes.  One thread per 16-byte chunk.
__global__ void block_w32_kernel(const bf16_t* __restrict__ Wvd, int64_t ldk, bf16_t* __restrict__ out, int64_t Vpad,
                                 int64_t dpad) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // destination chunk
    const int64_t ksteps = dpad / 32, total = Vpad * ksteps * 4;
    if (o >= total) return;
    const int64_t tile = o / (ksteps * 1024), rem = o % (ksteps * 1024);
    const int64_t ks = rem / 1024;
    const int within = (int)(rem % 1024), row = within >> 2, pos = within & 3;
    const int c = pos ^ ((row >> 2) & 3);
    const uint4 v = *(const uint4*)(Wvd + (tile * 256 + row) * ldk + ks * 32 + c * 8);
    *(uint4*)(out + o * 8) = v;
}

// ------------------------------------------------------------------------------------------ dz
template <class S>
__global__ __launch_bounds__(S::NT) void dz_kernel(DzArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.m0 >= Mr) return;
    const int tilesM = min(a.tilesM, (int)((Mr - a.m0 + S::BJ - 1) / S::BJ));   // row tiles that hold tokens
    for (int pid = blockIdx.x, ids = ids_for(a.tilesV, tilesM); pid < ids; pid += gridDim.x) {
    const TileId t = map_tile(pid, a.tilesV, tilesM, a.gi);
    if (!t.valid) continue;
    f32x16 acc[WI][WJ];
    mainloop<S>(a.Wvd + (int64_t)t.ti * S::BI * a.ldk, a.ldk,
                     a.Hc + (int64_t)t.tj * S::BJ * a.ldk, a.ldk, (int)(a.dpad / K_TILE), lds, acc);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the spare tile request of the last step
    __syncthreads();                                    // every wave is done with both stages
    // dz = -g p here; the +g of the sampled token's column is added by a separate small kernel, so
    // the per-element work is one fma, one exp, one multiply and half a convert.  Rows past the last
    // token get g = 0; columns past V hold finite values that only ever meet zero weights.
    const Lane<S> L;
    const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
    const int64_t jl_base = (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32);   // row in chunk
    const float zs = a.inv_temp * LOG2E;
    float ngj[WJ], nlse[WJ];
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int64_t j = a.m0 + jl_base + jb * 32 + L.lj;
        const bool live = j < M;
        ngj[jb] = live ? -a.rowg[j] * a.inv_temp : 0.f;
        nlse[jb] = live ? -a.lse_c[j] * LOG2E : 0.f;
    }
    store_tile_through_lds<S>(lds, L, a.dz + jl_base * a.ldz + i_base, a.ldz, [&](int ib, int jb, int v) {
        return ngj[jb] * __builtin_amdgcn_exp2f(fmaf(acc[ib][jb][v], zs, nlse[jb]));
    });
    }
}

// ------------------------------------------------------------------------------------------ dh
// The tiles of dHidden are long (the contraction runs over the whole vocabulary) and few: a launch has
// a handful of rounds of one tile per workgroup, and a last round that is only partly filled would
// leave most of the chip idle for a whole tile.  So the last, partial round of an XCD's share is not
// dealt out tile by tile: the contraction of each of its rem tiles is cut into S equal segments, and the
// rem x S (tile, segment) units are dealt out in short rounds, segment by segment, so that the workgroups
// of a short round are on the same K steps and share operand panels in the L2 as in a whole round.  A
// workgroup leaves the fp32 accumulators of a unit in `part`, and dh_reduce_kernel adds the S pieces of a
// tile in segment order and stores the result.  The last round then takes ceil(rem S / workgroups) / S of
// a tile's time, and the result does not depend on timing.
constexpr int DH_UNITS_PER_XCD = 64;   // partial tiles an XCD's last round may leave (dh_part_bytes)
struct DhShare {       // an XCD's share of the order, and how its last round is cut
    int total, per, wgs, mine, full_rounds, rem, segs;
    bool cut;
    __device__ __forceinline__ DhShare(int tilesD, int tilesM, int grid, int x, int ktiles, bool can_cut) {
        total = tilesD * tilesM; per = (total + 7) / 8; wgs = grid / 8;
        mine = max(0, min(per, total - x * per));
        full_rounds = mine / wgs; rem = mine - full_rounds * wgs;
        // the number of segments that makes the last round shortest: rounds(S) / S with rounds(S) = ceil(rem S / wgs)
        segs = 1;
        int best_rounds = 1;
        if (can_cut && rem > 0) {
            for (int sg = 2; sg <= 8 && sg <= ktiles && rem * sg <= DH_UNITS_PER_XCD; ++sg) {
                const int r = (rem * sg + wgs - 1) / wgs;
                if (r * segs < best_rounds * sg) { segs = sg; best_rounds = r; }
            }
        }
        // a cut costs a second pass over the partial tiles: it has to save a fifth of a tile's time at least
        cut = segs > 1 && best_rounds * 5 <= segs * 4;
        if (!cut) segs = 1;
    }
};

// stores a tile of dHidden: accumulators times the row factor (if any), bf16, to the rows' positions
template <class S>
__device__ __forceinline__ void dh_store(const DhArgs& a, const TileId& t, int M, const f32x16 (&acc)[S::WI][S::WJ]) {
    constexpr int WI = S::WI, WJ = S::WJ;
    const Lane<S> L;
    const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int64_t j = a.m0 + (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
        if (j >= M) continue;
        bf16_t* out = a.dhidden + (int64_t)a.row_index[j] * a.d;
        const float cj = a.rowc ? a.rowc[j] : 1.f;   // cached ratios: the row's -g p_y / temperature
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t i0 = i_base + ib * 32 + q * 8 + L.hi * 4;
                if (i0 < a.d)
                    *(uint2*)(out + i0) = pack_bf16x4(cj * acc[ib][jb][q * 4], cj * acc[ib][jb][q * 4 + 1],
                                                      cj * acc[ib][jb][q * 4 + 2], cj * acc[ib][jb][q * 4 + 3]);
            }
    }
}

// acc = the tile's contraction over the K steps [k0, k1)
template <class S, class Pace>
__device__ __forceinline__ void dh_contract(const DhArgs& a, const TileId& t, int k0, int k1, char* lds,
                                            f32x16 (&acc)[S::WI][S::WJ], Pace pace) {
    if (a.WdvB)   // A from the tile-blocked copy: one contiguous 128-byte-row block per K step
        mainloop<S, Pace>(a.WdvB + ((int64_t)t.ti * (a.Vpad / K_TILE) + k0) * (S::BI * 64), 64,
                          a.dz + (int64_t)t.tj * S::BJ * a.ldv + (int64_t)k0 * K_TILE, a.ldv, k1 - k0, lds, acc,
                          S::BI * 128, 128, pace);
    else
        mainloop<S, Pace>(a.Wdv + (int64_t)t.ti * S::BI * a.ldv + (int64_t)k0 * K_TILE, a.ldv,
                          a.dz + (int64_t)t.tj * S::BJ * a.ldv + (int64_t)k0 * K_TILE, a.ldv, k1 - k0, lds, acc, 128, 128, pace);
}

template <class S>
__global__ __launch_bounds__(S::NT) void dh_kernel(DhArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesD = (int)(a.dpadR / S::BI);
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.m0 >= Mr) return;
    // the order (and with it the split over the XCDs) covers the row tiles that hold tokens only: a
    // short last chunk would otherwise leave whole XCDs with nothing but empty tiles
    const int tilesM = min(a.tilesM, (int)((Mr - a.m0 + S::BJ - 1) / S::BJ));
    const int x = blockIdx.x & 7, w = blockIdx.x >> 3;
    const int ktiles = (int)(a.Vpad / K_TILE);
    const DhShare sh(tilesD, tilesM, gridDim.x, x, ktiles, a.part != nullptr && a.pace == nullptr);
    const int gi = a.gi > 0 ? a.gi : tilesD;
    // pacing of the launch's workgroups (see GridPace): with total = 8 * per tiles (or fewer in the last
    // XCD shares) the workgroups of round r are those whose id is a valid tile
    GridPace pace{a.pace, 0u, 0u, a.pace ? a.pace_every : 0};
    unsigned before = 0;   // valid tiles of the rounds before this one, over all XCDs
    // rounds dealt out tile by tile: uniform over the launch when pacing is on (nobody cuts then)
    const int whole_rounds = sh.cut ? sh.full_rounds : (pace.every ? (sh.per + sh.wgs - 1) / sh.wgs : (sh.mine + sh.wgs - 1) / sh.wgs);
    for (int round = 0; round < whole_rounds; ++round) {
        const int pos = round * sh.wgs + w;
        unsigned now = 0;
        if (pace.every) {
            for (int xx = 0; xx < 8; ++xx) {
                const int mine = max(0, min(sh.per, sh.total - xx * sh.per));
                now += (unsigned)max(0, min(sh.wgs, mine - round * sh.wgs));
            }
        }
        if (pos >= sh.mine) { before += now; continue; }
        const TileId t = tile_of_vid(x * sh.per + pos, tilesD, tilesM, gi);
        f32x16 acc[WI][WJ];
        pace.n = now;
        pace.base = (unsigned)(ktiles / (pace.every ? pace.every : 1)) * before;
        before += now;
        dh_contract<S, GridPace>(a, t, 0, ktiles, lds, acc, pace);
        dh_store<S>(a, t, M, acc);
    }
    if (!sh.cut) return;
    // the last round: unit u = (segment u / rem, tile u % rem), dealt out in rounds of one unit per workgroup;
    // its accumulators go to part[x * DH_UNITS_PER_XCD + u]
    for (int u = w; u < sh.rem * sh.segs; u += sh.wgs) {
        const int seg = u / sh.rem, tpos = u - seg * sh.rem;
        const int k0 = (int)((int64_t)ktiles * seg / sh.segs), k1 = (int)((int64_t)ktiles * (seg + 1) / sh.segs);
        const TileId t = tile_of_vid(x * sh.per + sh.full_rounds * sh.wgs + tpos, tilesD, tilesM, gi);
        f32x16 acc[WI][WJ];
        dh_contract<S, NoPace>(a, t, k0, k1, lds, acc, NoPace());
        // the accumulators as they are: register r of thread tid at part[unit slot][r][tid]
        int64_t off = ((int64_t)x * DH_UNITS_PER_XCD + u) * (S::BI * S::BJ) + threadIdx.x;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib)
#pragma unroll
            for (int jb = 0; jb < WJ; ++jb) {
                asm volatile("" : "+v"(off));   // one address per block of 16 stores, formed here and not ahead of the loops
#pragma unroll
                for (int v = 0; v < 16; ++v) a.part[off + v * S::NT] = acc[ib][jb][v];
                off += 16 * S::NT;
            }
    }
}

// adds the pieces of the tiles that dh_kernel cut (same launch geometry: grid_of_dh says how many
// workgroups that launch had) and stores them; one workgroup per (XCD, tile of its last round)
template <class S>
__global__ __launch_bounds__(S::NT) void dh_reduce_kernel(DhArgs a, int grid_of_dh) {
    constexpr int WI = S::WI, WJ = S::WJ;
    const int tilesD = (int)(a.dpadR / S::BI);
    const int M = a.counts[CNT_M], Mr = a.counts[CNT_MR];
    if (a.m0 >= Mr) return;
    const int tilesM = min(a.tilesM, (int)((Mr - a.m0 + S::BJ - 1) / S::BJ));
    const int x = blockIdx.x & 7, tpos = blockIdx.x >> 3;
    const int ktiles = (int)(a.Vpad / K_TILE);
    const DhShare sh(tilesD, tilesM, grid_of_dh, x, ktiles, true);
    if (!sh.cut || tpos >= sh.rem) return;
    const TileId t = tile_of_vid(x * sh.per + sh.full_rounds * sh.wgs + tpos, tilesD, tilesM, a.gi > 0 ? a.gi : tilesD);
    // One 32 x 32 block at a time, its pieces added in segment order (a fixed order of summation).  The 16
    // loads of a piece are independent and in flight together; with all 256 accumulators of the tile live at
    // once the loads went out one by one, each a trip to memory, and a tile with five pieces took 3 ms.
    const Lane<S> L;
    const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
#pragma unroll
    for (int jb = 0; jb < WJ; ++jb) {
        const int64_t j = a.m0 + (int64_t)t.tj * S::BJ + L.wave_j * (WJ * 32) + jb * 32 + L.lj;
        const bool row_live = j < M;
        bf16_t* out = a.dhidden + (row_live ? (int64_t)a.row_index[j] * a.d : 0);
        const float cj = (a.rowc && row_live) ? a.rowc[j] : 1.f;
#pragma unroll
        for (int ib = 0; ib < WI; ++ib) {
            float sum[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[v] = 0.f;
            for (int seg = 0; seg < sh.segs; ++seg) {
                const float* in = a.part + ((int64_t)x * DH_UNITS_PER_XCD + seg * sh.rem + tpos) * (S::BI * S::BJ) + threadIdx.x +
                                  (int64_t)((ib * WJ + jb) * 16) * S::NT;
                float got[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) got[v] = in[v * S::NT];
#pragma unroll
                for (int v = 0; v < 16; ++v) sum[v] += got[v];
            }
            if (!row_live) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t i0 = i_base + ib * 32 + q * 8 + L.hi * 4;
                if (i0 < a.d)
                    *(uint2*)(out + i0) = pack_bf16x4(cj * sum[q * 4], cj * sum[q * 4 + 1], cj * sum[q * 4 + 2], cj * sum[q * 4 + 3]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ dw
template <class S, bool DEEP = false>
__global__ __launch_bounds__(S::NT) void dw_kernel(DwArgs a) {
    constexpr int WI = S::WI, WJ = S::WJ;
    extern __shared__ __attribute__((aligned(128))) char lds[];
    const int tilesV = (int)(a.Vpad / S::BI), tilesD = (int)(a.dpadR / S::BJ);
    const int Mr = a.counts[CNT_MR];
    int64_t rows = (int64_t)Mr - a.m0;
    rows = rows < 0 ? 0 : (rows > a.Mc ? a.Mc : rows);
    if (rows == 0 && a.beta) return;   // nothing to add
    for (int pid = blockIdx.x, ids = ids_for(tilesV, tilesD); pid < ids; pid += gridDim.x) {
    const TileId t = map_tile(pid, tilesV, tilesD, a.gi);
    if (!t.valid) continue;
    f32x16 acc[WI][WJ];
    if constexpr (DEEP)
        mainloop_kmajor32<S, 4>(a.dz + (int64_t)t.ti * S::BI, a.ldz, a.Hc + (int64_t)t.tj * S::BJ, a.ldH, (int)(rows / 32), lds, acc);
    else
        mainloop_kmajor<S>(a.dz + (int64_t)t.ti * S::BI, a.ldz, a.Hc + (int64_t)t.tj * S::BJ, a.ldH,
                           (int)(rows / K_TILE), lds, acc);
    const Lane<S> L;
    const int64_t i_base = (int64_t)t.ti * S::BI + L.wave_i * (WI * 32);
    const bool vec = (a.V % 4) == 0;
    const float bs = (a.beta && a.beta_scale) ? a.beta_scale[0] : 1.f;   // what the sum so far is multiplied by
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
                        *(float4*)p = make_float4(cur.x * bs + o[0], cur.y * bs + o[1], cur.z * bs + o[2], cur.w * bs + o[3]);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (i0 + r < a.V) p[r] = (a.beta ? p[r] * bs : 0.f) + o[r];
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (i0 + r < a.V) {
                            float* p = a.dW + (i0 + r) * a.d + jd;
                            *p = (a.beta ? *p * bs : 0.f) + o[r];
                        }
                }
            }
    }
    }
}

// Logit of the sampled token: zy[j] = inv_temp * <Hc[j, :], Wvd[tok_j, :]>, one wave per token row
// (16-byte loads, fp32 accumulation, fixed reduction tree).
// If refz is given it receives the reference of the storing forward: zy[j] - ref_logp[row_index[j]]
// (zy[j] alone without ref_logp or where that value is not finite).
__global__ __launch_bounds__(256) void token_logit_kernel(const bf16_t* __restrict__ Hc, const bf16_t* __restrict__ Wvd,
                                                          int64_t ldk, int64_t dpad, const int32_t* __restrict__ tokc,
                                                          const int32_t* __restrict__ counts, float inv_temp,
                                                          float* __restrict__ zy, const float* __restrict__ ref_logp,
                                                          const int32_t* __restrict__ row_index,
                                                          float* __restrict__ refz, int64_t row0) {
    const int64_t j = row0 + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
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
    if (lane == 0) {
        const float z = acc * inv_temp;
        zy[j] = z;
        if (refz) {
            float lb = ref_logp ? ref_logp[row_index[j]] : 0.f;
            if (!isfinite(lb)) lb = 0.f;
            refz[j] = z - lb;
        }
    }
}

// dz[row][tok_row] += g: the one-hot part of dz = g (onehot - p)
__global__ void token_onehot_kernel(bf16_t* __restrict__ dz, int64_t ldz, int64_t m0, int64_t rows,
                                    const int32_t* __restrict__ tokc, const float* __restrict__ rowg, float inv_temp,
                                    const int32_t* __restrict__ counts) {
    const int64_t jl = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t j = m0 + jl;
    if (jl >= rows || j >= counts[CNT_M]) return;
    bf16_t* p = dz + jl * ldz + tokc[j];
    const float cur = (float)__builtin_bit_cast(__bf16, *p);
    const __bf16 r = (__bf16)(cur + rowg[j] * inv_temp);
    *p = __builtin_bit_cast(bf16_t, r);
}

// After a forward that stored u = exp(z - r) (see fwd_lse_kernel), with lse and the row coefficients
// g known: dz[j][v] = (g_j / temperature) (onehot_y[v] - p_v) = c_j u'[j][v], with the row factor
// c_j = -(g_j / temperature) exp(r_j - lse_j) and u' = u except at the sampled token, where
// u'[j][y] = exp(lse_j - r_j) (p_y - 1).  One wave per token row writes c_j (0 past the last
// token), replaces that one element, and scales the row of the packed hidden copy by c_j: dW
// contracts over token rows, so there the factor has to sit on an operand (dHidden applies it to
// its accumulators).  |lse - r| is clamped at 80 (sets RAPID_STATUS_LOGIT_RANGE: such a row's
// gradient is truncated).
__global__ __launch_bounds__(256) void cache_finish_kernel(bf16_t* __restrict__ u, int64_t ldz, bf16_t* __restrict__ Hc,
                                                           int64_t ldk, const int32_t* __restrict__ tokc,
                                                           const float* __restrict__ zy, const float* __restrict__ refz,
                                                           const float* __restrict__ lse_c, const float* __restrict__ rowg,
                                                           float inv_temp, const int32_t* __restrict__ counts,
                                                           int64_t row0, float* __restrict__ rowc,
                                                           int32_t* __restrict__ dev_status) {
    const int64_t j = row0 + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int M = counts[CNT_M], Mr = counts[CNT_MR];
    if (j >= Mr) return;
    float c = 0.f;
    if (j < M) {
        const float lse = lse_c[j];
        float a = lse - refz[j];
        if (!(fabsf(a) <= 80.f)) {
            a = a > 0.f ? 80.f : -80.f;
            if (lane == 0 && dev_status) atomicOr(dev_status, RAPID_STATUS_LOGIT_RANGE);
        }
        c = -rowg[j] * inv_temp * __expf(-a);
        if (lane == 0) {
            const __bf16 r = (__bf16)(__expf(a) * expm1f(zy[j] - lse));   // exp(lse - r) (p_y - 1)
            u[(j - row0) * ldz + tokc[j]] = __builtin_bit_cast(bf16_t, r);
        }
    }
    if (lane == 0) rowc[j] = c;
    uint4* row = (uint4*)(Hc + j * ldk);
    for (int c8 = lane; c8 < ldk / 8; c8 += 64) {
        const uint4 in = row[c8];
        const uint32_t w[4] = {in.x, in.y, in.z, in.w};
        float o[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[2 * e] = c * __builtin_bit_cast(float, w[e] << 16);
            o[2 * e + 1] = c * __builtin_bit_cast(float, w[e] & 0xffff0000u);
        }
        const uint2 a0 = pack_bf16x4(o[0], o[1], o[2], o[3]), a1 = pack_bf16x4(o[4], o[5], o[6], o[7]);
        row[c8] = make_uint4(a0.x, a0.y, a1.x, a1.y);
    }
}

// Lets `kernel` use `bytes` of dynamic LDS: once per kernel and device (the attribute belongs to the
// device's copy of the function), not once per launch.  One static bit mask per kernel.
template <auto kernel>
void allow_lds(int bytes) {
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    (void)hipGetDevice(&dev);
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return;
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess)
        done.fetch_or(bit, std::memory_order_release);
}

// waves per workgroup: 4 (2 x 2 of 128 x 128), 8 (2 x 4 of 128 x 64) or 16; 0 = each kernel's own
// default: 8 for the logits kernels and dW, 4 for dHidden (measured: its long K loop gains more from
// the 4-wave tile's third fewer LDS reads than it loses in latency hiding)
std::atomic<int> g_waves{0};
static int waves_for(int own_default) {
    const int w = g_waves.load();
    return w ? w : own_default;
}

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
    if (a.zc) {
        allow_lds<&fwd_lse_kernel<S, true>>(S::LDS_BYTES);
        fwd_lse_kernel<S, true><<<grid_for(a.tilesV, a.tilesM), S::NT, S::LDS_BYTES, st>>>(a);
    } else {
        allow_lds<&fwd_lse_kernel<S, false>>(S::LDS_BYTES);
        fwd_lse_kernel<S, false><<<grid_for(a.tilesV, a.tilesM), S::NT, S::LDS_BYTES, st>>>(a);
    }
}
template <class S>
void launch_dz_t(const DzArgs& a, hipStream_t st) {
    allow_lds<&dz_kernel<S>>(S::LDS_BYTES);
    dz_kernel<S><<<grid_for(a.tilesV, a.tilesM), S::NT, S::LDS_BYTES, st>>>(a);
}
template <class S>
void launch_dh_t(const DhArgs& a, hipStream_t st) {
    allow_lds<&dh_kernel<S>>(S::LDS_BYTES);
    const unsigned grid = grid_for((int)(a.dpadR / S::BI), a.tilesM);
    DhArgs b = a;
    // a cut last round needs DH_UNITS_PER_XCD tiles of fp32 scratch per XCD and whole XCD shares of workgroups
    if (grid % 8 != 0 || grid < 16 || (size_t)8 * DH_UNITS_PER_XCD * S::BI * S::BJ * 4 > a.part_bytes) b.part = nullptr;
    dh_kernel<S><<<grid, S::NT, S::LDS_BYTES, st>>>(b);
    if (b.part && !b.pace) dh_reduce_kernel<S><<<grid, S::NT, 0, st>>>(b, (int)grid);
}
template <class S, bool DEEP = false>
void launch_dw_t(const DwArgs& a, hipStream_t st) {
    allow_lds<&dw_kernel<S, DEEP>>(S::LDS_BYTES);
    dw_kernel<S, DEEP><<<grid_for((int)(a.Vpad / S::BI), (int)(a.dpadR / S::BJ)), S::NT, S::LDS_BYTES, st>>>(a);
}

}  // namespace

// DH_UNITS_PER_XCD fp32 tiles of 256 x 256 for each of the 8 XCDs
size_t dh_part_bytes() { return (size_t)8 * DH_UNITS_PER_XCD * 256 * 256 * 4; }
void set_waves_per_workgroup(int n) { g_waves = (n == 4 || n == 8 || n == 16) ? n : 0; }
void set_cu_count(int n) { g_num_cu = n >= 8 ? n : 8; }


void launch_block_w32(const bf16_t* Wvd, int64_t ldk, bf16_t* out, int64_t Vpad, int64_t dpad, hipStream_t st) {
    const int64_t chunks = Vpad * (dpad / 32) * 4;
    block_w32_kernel<<<(unsigned)((chunks + 255) / 256), 256, 0, st>>>(Wvd, ldk, out, Vpad, dpad);
}
void launch_fwd_lse(const FwdArgs& a, hipStream_t st) {
    if (a.WvdB && a.k32_mode == 3) {   // one workgroup of 4 waves per CU, K steps of 32 requested three steps ahead
        const unsigned grid = grid_for(a.tilesV, a.tilesM);
        if (a.zc) {
            allow_lds<&fwd_lse2_kernel<Fwd4, true>>(Fwd4::LDS_BYTES);
            fwd_lse2_kernel<Fwd4, true><<<grid, 256, Fwd4::LDS_BYTES, st>>>(a);
        } else {
            allow_lds<&fwd_lse2_kernel<Fwd4, false>>(Fwd4::LDS_BYTES);
            fwd_lse2_kernel<Fwd4, false><<<grid, 256, Fwd4::LDS_BYTES, st>>>(a);
        }
        return;
    }
    if (a.WvdB && a.k32_mode == 2) {   // one workgroup of 8 waves per CU, K steps of 32 requested three steps ahead
        const unsigned grid = grid_for(a.tilesV, a.tilesM);
        if (a.zc) {
            allow_lds<&fwd_lse2_kernel<Fwd3, true>>(Fwd3::LDS_BYTES);
            fwd_lse2_kernel<Fwd3, true><<<grid, 512, Fwd3::LDS_BYTES, st>>>(a);
        } else {
            allow_lds<&fwd_lse2_kernel<Fwd3, false>>(Fwd3::LDS_BYTES);
            fwd_lse2_kernel<Fwd3, false><<<grid, 512, Fwd3::LDS_BYTES, st>>>(a);
        }
        return;
    }
    if (a.WvdB) {   // two workgroups of 4 waves per CU on 256 x 128 tiles
        const int ids = ids_for(a.tilesV, a.tilesM * 2), slots = g_num_cu.load() / 8 * 8 * 2;
        const unsigned grid = (unsigned)(ids < slots ? ids : slots);
        if (a.zc) {
            allow_lds<&fwd_lse2_kernel<Fwd2, true>>(Fwd2::LDS_BYTES);
            fwd_lse2_kernel<Fwd2, true><<<grid, 256, Fwd2::LDS_BYTES, st>>>(a);
        } else {
            allow_lds<&fwd_lse2_kernel<Fwd2, false>>(Fwd2::LDS_BYTES);
            fwd_lse2_kernel<Fwd2, false><<<grid, 256, Fwd2::LDS_BYTES, st>>>(a);
        }
        return;
    }
    const int w = waves_for(8);
    if (w == 16) launch_fwd_lse_t<G16>(a, st); else if (w == 8) launch_fwd_lse_t<G8>(a, st); else launch_fwd_lse_t<G4>(a, st);
}
void launch_token_logit(const FwdArgs& a, int64_t row0, int64_t rows_max, hipStream_t st) {
    if (rows_max <= 0) return;
    token_logit_kernel<<<(unsigned)((rows_max + 3) / 4), 256, 0, st>>>(a.Hc, a.Wvd, a.ldk, a.dpad, a.tokc, a.counts,
                                                                     a.inv_temp, a.zy, a.ref_logp, a.row_index,
                                                                     a.zc ? a.refz : nullptr, row0);
}
int fwd_slots_per_tile() { return 2; }

void launch_dz(const DzArgs& a, hipStream_t st) {
    const int w = waves_for(8);
    if (w == 16) launch_dz_t<G16>(a, st); else if (w == 8) launch_dz_t<G8>(a, st); else launch_dz_t<G4>(a, st);
    const int64_t rows = (int64_t)a.tilesM * 256;
    token_onehot_kernel<<<(unsigned)((rows + 255) / 256), 256, 0, st>>>(a.dz, a.ldz, a.m0, rows, a.tokc, a.rowg,
                                                                      a.inv_temp, a.counts);
}

void launch_cache_finish(bf16_t* u, int64_t ldz, bf16_t* Hc, int64_t ldk, const int32_t* tokc,
                         const float* zy, const float* refz, const float* lse_c, const float* rowg, float inv_temp,
                         const int32_t* counts, int64_t row0, int64_t rows_max, float* rowc, int32_t* dev_status,
                         hipStream_t st) {
    if (rows_max <= 0) return;
    cache_finish_kernel<<<(unsigned)((rows_max + 3) / 4), 256, 0, st>>>(u, ldz, Hc, ldk, tokc, zy, refz, lse_c, rowg,
                                                                        inv_temp, counts, row0, rowc, dev_status);
}
void launch_dh(const DhArgs& a, hipStream_t st) {
    const int w = waves_for(4);
    if (a.dpadR % 256 == 0) {
        if (w == 16) launch_dh_t<G16>(a, st); else if (w == 8) launch_dh_t<G8>(a, st); else launch_dh_t<G4>(a, st);
    } else {   // d padded to a multiple of 128 only
        if (w == 16) launch_dh_t<G16_I128>(a, st); else if (w == 8) launch_dh_t<G8_I128>(a, st); else launch_dh_t<G4_I128>(a, st);
    }
}

std::atomic<int> g_dw_deep{0};
void set_dw_deep(int on) { g_dw_deep = on ? 1 : 0; }
void launch_dw(const DwArgs& a, hipStream_t st) {
    const int w = waves_for(8);
    if (g_dw_deep.load() && w == 8) {   // K steps of 32 rows, requests three steps ahead
        if (a.dpadR % 256 == 0) launch_dw_t<G8, true>(a, st); else launch_dw_t<G8_J128, true>(a, st);
        return;
    }
    if (a.dpadR % 256 == 0) {
        if (w == 16) launch_dw_t<G16>(a, st); else if (w == 8) launch_dw_t<G8>(a, st); else launch_dw_t<G4>(a, st);
    } else {   // d padded to a multiple of 128 only
        if (w == 16) launch_dw_t<G16_J128>(a, st); else if (w == 8) launch_dw_t<G8_J128>(a, st); else launch_dw_t<G4_J128>(a, st);
    }
}

}  // namespace rapid
