// Host side of the C ABI declared in rapid.h: argument validation, workspace planning and the
// order of kernel launches.  No device memory is allocated here and nothing synchronises.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <cmath>
#include <mutex>

#include "rapid_internal.h"
#include "rapid_tuning.h"

// Scratch of rapid_logprob_fwd_static, the entry point for callers that cannot allocate device
// memory.  Every GPU the library is used on holds its own copy at its own address from the moment
// this code object is loaded there until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress: the per-device address it returns is what kernels and fills are given.
#define RAPID_STATIC_SCRATCH_BYTES ((size_t)768 << 20)
static __device__ __align__(256) unsigned char scratch[RAPID_STATIC_SCRATCH_BYTES];

namespace rapid {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

namespace {


// tuning switches (rapid_tuning.h): one atomic word each, so that a change made by another thread is
// seen whole
std::atomic<int> g_gi_fwd{4}, g_gi_dh{0}, g_gi_dw{2};   // L2 blocking of the tile order (tuning keys 10..12)
std::atomic<int> g_blocked_wdv{1};            // dH reads W from a tile-blocked copy (tuning key 14)
std::atomic<int> g_probe_cus{256};            // compute units of the current device
std::atomic<int> g_cached_dw_step_tiles{0};   // row tiles per dW launch with the cache (tuning key 20; 0 = all rows of the chunk)
std::atomic<int> g_cached_step_tiles{256};    // row tiles per dHidden / dW launch with the cache (tuning key 15; 0 = all rows)
std::atomic<int> g_pace_every{0};             // K steps between meetings of the dHidden workgroups (tuning key 16; 0 = off)
std::atomic<int> g_fwd_block_tiles{64};       // row tiles per launch of the two logits kernels (tuning key 13)
std::atomic<int> g_fwd_two_wg{0};             // logits kernels: two 4-wave workgroups per CU on 256 x 128 tiles (tuning key 21)
std::atomic<int> g_skip_idle{1};              // cached backward: generations without gradient are left out of dHidden / dW (tuning key 19)
std::atomic<int> g_dh_split{1};               // dHidden cuts the tiles of a partly filled last round along the contraction (tuning key 17)

// address of `scratch` on each device, looked up once per device with that device current
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        set_error("hipGetDevice failed, or device index beyond %d", MAX_DEVICES - 1);
        return RAPID_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_error("hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
            return RAPID_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RAPID_OK;
}

// Optional per-stage timing with HIP events on the caller's stream (off by default).
enum Stage { ST_COMPACT = 0, ST_PACK, ST_FWD_LSE, ST_MERGE, ST_ESTIMATOR, ST_ZERO, ST_DZ, ST_DZ_T, ST_DH, ST_DW,
             ST_F32, ST_CONVERT, ST_COUNT };
struct Profiler {
    bool on = false;
    static constexpr int MAX_SPANS = 8192;
    hipEvent_t ev[2 * MAX_SPANS];
    int stage[MAX_SPANS];
    int created = 0, used = 0;
    void begin(int st_id, hipStream_t st) {
        if (!on || used >= MAX_SPANS) return;
        while (created < 2 * (used + 1)) {
            if (hipEventCreate(&ev[created]) != hipSuccess) { on = false; return; }
            ++created;
        }
        stage[used] = st_id;
        (void)hipEventRecord(ev[2 * used], st);
    }
    void end(hipStream_t st) {
        if (!on || used >= MAX_SPANS) return;
        (void)hipEventRecord(ev[2 * used + 1], st);
        ++used;
    }
};
Profiler g_prof;
struct Span {
    hipStream_t st;
    Span(int id, hipStream_t s) : st(s) { g_prof.begin(id, s); }
    ~Span() { g_prof.end(st); }
};

struct Plan {
    int op, dtype;
    int64_t N, T, d, V, K;
    int64_t Mmax, Mmax_pad, dpad, dpadR, Vpad;
    int64_t ldk, ldv;   // leading dimensions of the [*, dpad] and [*, Vpad] operands
    int P;              // log-sum-exp partial slots per row
    int64_t Mc;         // rows per backward chunk (f32: also per forward chunk)
    // Cached backward: the compact rows come in Cmax regions of Rcap rows, one per chunk of whole groups
    // (Mmax_pad = Cmax * Rcap then); the cache and the log-sum-exp partials hold one region.  Cmax = 0 otherwise.
    int64_t Rcap;
    int Cmax;
    bool two_wg;        // the forward runs two workgroups per CU and reads W from its K-blocked copy (Wvd32)
    int64_t ld_part;    // columns of the log-sum-exp partials
    int64_t rms_blocks; // row blocks of the final norm's dweight partial sums
    size_t per_row;     // chunk bytes per row
    size_t fixed, total;
    // offsets into the workspace
    size_t counts, pace, seq_len, cu, row_index, tokc, seqc, zy, refz, lse_c, inv_rms, rms_part, rowc, rowg, logp_tmp, s64, s32, adv, adv64, g, g64, tsum, tmax,
        Hc, Wvd, Wdv, WdvB, dh_part, part_max, part_sum, dw32, chunk0, tab, gen_row0, gen_chunk, gseen, lam_state, lam_chunk, beta_scale, idle, len_live, cu_live, live_group, gruns, Wvd32;
};

size_t take(size_t& cur, size_t bytes) {
    const size_t at = cur;
    cur += (bytes + 255) / 256 * 256;
    return at;
}

// lays the workspace out; chunk sizing is done by the caller through `avail`.  Cmax > 0: the layout of the
// cached backward with Cmax regions of Rcap rows (bf16, RAPID_OP_IW_PG_FWD_BWD only).
bool make_plan(Plan& p, int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype, int64_t Rcap = 0,
               int Cmax = 0) {
    memset(&p, 0, sizeof(p));
    if (N <= 0 || T <= 0 || d <= 0 || V <= 0) return false;
    if (dtype != RAPID_DTYPE_F32 && dtype != RAPID_DTYPE_BF16) return false;
    // limits: positions and generations fit int32 indices; V keeps every two-dimensional launch inside the
    // 65535-block limit of the second grid dimension (V / 64 blocks in the transposing pack)
    if (N * T > (int64_t)2000000000 || V > (int64_t)4000000 || d > 65536 || N > (int64_t)2000000000)
        return false;
    if (op == RAPID_OP_IW_PG_FWD_BWD && K <= 0) return false;
    p.op = op; p.dtype = dtype; p.N = N; p.T = T; p.d = d; p.V = V; p.K = K;
    p.Mmax = N * T;
    p.Mmax_pad = Cmax > 0 ? (int64_t)Cmax * Rcap : round_up(p.Mmax, ROW_TILE);
    p.Rcap = Rcap; p.Cmax = Cmax;
    p.ld_part = Cmax > 0 ? Rcap : p.Mmax_pad;
    if (p.Mmax_pad > (int64_t)2100000000) return false;   // compact row indices are int32
    p.dpad = round_up(d, K_TILE);
    // dHidden / dW tile d by 256 when that pads by at most a sixth (full-size tiles beat the padding),
    // else by 128
    p.dpadR = (round_up(d, 256) - d) * 6 <= d ? round_up(d, 256) : round_up(d, 128);
    p.Vpad = round_up(V, 256);
    p.ldk = padded_ld(p.dpadR);   // >= dpad; the dW kernel reads whole 128-column tiles of Hc
    p.ldv = padded_ld(p.Vpad);
    p.P = (int)(p.Vpad / 256) * fwd_slots_per_tile();
    const bool bwd = op == RAPID_OP_IW_PG_FWD_BWD;
    size_t cur = 0;
    p.counts = take(cur, CNT_WORDS * 4);
    p.pace = take(cur, 64 * 4);
    p.seq_len = take(cur, (size_t)N * 4);
    p.cu = take(cur, (size_t)(N + 1) * 4);
    p.row_index = take(cur, (size_t)p.Mmax_pad * 4);
    p.tokc = take(cur, (size_t)p.Mmax_pad * 4);
    p.seqc = take(cur, (size_t)p.Mmax_pad * 4);
    p.zy = take(cur, (size_t)p.Mmax_pad * 4);
    p.refz = take(cur, (size_t)p.Mmax_pad * 4);
    p.lse_c = take(cur, (size_t)p.Mmax_pad * 4);
    if (dtype == RAPID_DTYPE_BF16) p.inv_rms = take(cur, (size_t)p.Mmax_pad * 4);   // final-norm option
    if (bwd) {
        p.rowc = take(cur, (size_t)p.Mmax_pad * 4);
        p.rms_blocks = Cmax > 0 ? (int64_t)Cmax * rmsnorm_dweight_blocks(Rcap) : rmsnorm_dweight_blocks(p.Mmax_pad);
        if (dtype == RAPID_DTYPE_BF16) p.rms_part = take(cur, (size_t)p.rms_blocks * d * 4);
        p.rowg = take(cur, (size_t)p.Mmax_pad * 4);
        p.adv64 = take(cur, (size_t)N * 8);
        p.gruns = take(cur, (size_t)(3 * K + 1) * 4);
        if (dtype == RAPID_DTYPE_BF16) {   // the chunk plan; without the cache the whole batch is its one chunk
            p.tab = take(cur, (size_t)(Cmax > 0 ? Cmax : 1) * CH_WORDS * 4);
            p.gen_row0 = take(cur, (size_t)N * 4);
            p.gen_chunk = take(cur, (size_t)N * 4);
            p.gseen = take(cur, (size_t)K * 4);
            p.idle = take(cur, (size_t)N * 4);
            p.len_live = take(cur, (size_t)N * 4);
            p.cu_live = take(cur, (size_t)(N + 1) * 4);
            p.live_group = take(cur, (size_t)K * 4);
        }
        if (Cmax > 0) {
            p.lam_state = take(cur, 2 * 8);
            p.lam_chunk = take(cur, (size_t)Cmax * 8);
            p.beta_scale = take(cur, 64);
        }
        p.g64 = take(cur, (size_t)N * 8);
        p.tsum = take(cur, (size_t)N * 8);
        p.tmax = take(cur, (size_t)N * 8);
        p.logp_tmp = take(cur, (size_t)p.Mmax * 4);
        p.s64 = take(cur, (size_t)N * 8);
        p.s32 = take(cur, (size_t)N * 4);
        p.adv = take(cur, (size_t)N * 4);
        p.g = take(cur, (size_t)N * 4);
        p.dw32 = take(cur, (size_t)d * V * 4);
    }
    if (dtype == RAPID_DTYPE_BF16) {
        p.Hc = take(cur, (size_t)p.Mmax_pad * p.ldk * 2);
        p.Wvd = take(cur, (size_t)p.Vpad * p.ldk * 2);
        p.two_wg = g_fwd_two_wg.load() != 0;
        if (p.two_wg) p.Wvd32 = take(cur, (size_t)p.Vpad * p.dpad * 2);
        p.part_max = take(cur, (size_t)p.P * p.ld_part * 4);
        p.part_sum = take(cur, (size_t)p.P * p.ld_part * 4);
        if (bwd) {
            p.Wdv = take(cur, (size_t)p.dpadR * p.ldv * 2);
            p.WdvB = take(cur, (size_t)p.dpadR * p.Vpad * 2);
            p.dh_part = take(cur, dh_part_bytes());
            p.per_row = (size_t)p.ldv * 2;   // the dz chunk
        }
    } else {
        p.per_row = (size_t)V * 4;                // logits / dz chunk
    }
    p.fixed = cur;
    return true;
}

void size_chunks(Plan& p, int64_t Mc) {
    Mc = Mc / ROW_TILE * ROW_TILE;
    if (Mc < ROW_TILE) Mc = ROW_TILE;
    if (Mc > p.Mmax_pad) Mc = p.Mmax_pad;
    if (p.Cmax > 0) Mc = p.Rcap;   // the cache holds one region
    p.Mc = Mc;
    size_t cur = p.fixed;
    if (p.per_row) {
        if (p.dtype == RAPID_DTYPE_BF16) {
            p.chunk0 = take(cur, (size_t)Mc * p.ldv * 2);
        } else {
            p.chunk0 = take(cur, (size_t)Mc * p.V * 4);
        }
    }
    p.total = cur;
}

// rows the cache must hold: the caller's bound on the number of valid tokens (0 = none given), at most N*T
int64_t cache_rows(const Plan& p, int64_t max_tokens) {
    const int64_t t = (max_tokens > 0 && max_tokens < p.Mmax) ? max_tokens : p.Mmax;
    return round_up(t, ROW_TILE);
}

int64_t recommended_chunk(const Plan& p) { return p.dtype == RAPID_DTYPE_BF16 ? 65536 : 4096; }

// Chunks the cached backward may need when the cache holds Rcap rows and the batch at most `rows` tokens:
// chunks are filled greedily with whole groups, so two consecutive chunks together hold more than Rcap
// tokens (the first group of the second did not fit into the first), hence at most 2 floor(rows / Rcap) + 1.
int cached_chunks(int64_t rows, int64_t Rcap) { return Rcap >= rows ? 1 : (int)(2 * (rows / Rcap) + 1); }

// Cache rows of the recommended workspace, if the batch has more (tuning key 18).  Every launch of the dHidden and
// dW kernels ends in a tail (workgroups finish at different times; dW re-reads and re-writes all of dW), so fewer,
// larger chunks are faster: measured at the 1.5B shape, 65536 rows 338.7 ms per call (24.8 GiB), 90112 rows 334.4 ms
// (31.7 GiB), 98304 rows 331.7 ms (34.3 GiB), the whole batch at once 329 ms (91 GiB).
std::atomic<int> g_cached_rcap{90112};

// workspace bytes of the cached backward with a cache of Rcap rows for a batch of at most `rows` tokens; 0 if invalid
size_t cached_total(int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int64_t rows, int64_t Rcap, Plan* out = nullptr) {
    Plan p;
    if (Rcap > rows) Rcap = rows;
    if (!make_plan(p, RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, RAPID_DTYPE_BF16, Rcap, cached_chunks(rows, Rcap))) return 0;
    size_chunks(p, Rcap);
    if (out) *out = p;
    return p.total + 1024;
}

// Cache rows a call with this workspace works with: every row of the batch if that fits (one chunk), otherwise the
// largest window that does; 0 if not even one row tile fits.  Fills `out` with the plan of that geometry.
int64_t choose_cache(int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int64_t rows, size_t workspace_bytes, Plan* out) {
    size_t need = cached_total(N, T, d, V, K, rows, rows, out);
    if (need != 0 && need <= workspace_bytes) return rows;
    int64_t lo = 1, hi = rows / ROW_TILE - 1, best = 0;     // cache rows in row tiles
    while (lo <= hi) {
        const int64_t mid = (lo + hi) / 2;
        need = cached_total(N, T, d, V, K, rows, mid * ROW_TILE);
        if (need != 0 && need <= workspace_bytes) { best = mid; lo = mid + 1; } else { hi = mid - 1; }
    }
    // the size is not monotone everywhere (the number of regions steps down as the cache grows)
    while (best > 0 && ((need = cached_total(N, T, d, V, K, rows, best * ROW_TILE, out)) == 0 || need > workspace_bytes))
        --best;
    return best * ROW_TILE;
}

// largest chunk that fits into `avail` bytes; 0 if even the minimum does not
int64_t fit_chunk(const Plan& p, size_t avail) {
    if (!p.per_row) return avail >= p.fixed ? ROW_TILE : 0;
    if (avail < p.fixed + 1024) return 0;
    int64_t Mc = (int64_t)((avail - p.fixed - 1024) / p.per_row) / ROW_TILE * ROW_TILE;
    if (Mc > p.Mmax_pad) Mc = p.Mmax_pad;
    return Mc;
}

int check_arch() {
    static thread_local int cached_dev = -1, cached_rc = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        set_error("hipGetDevice failed");
        return RAPID_ERR_HIP;
    }
    if (dev == cached_dev) return cached_rc;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        set_error("hipGetDeviceProperties failed");
        return RAPID_ERR_HIP;
    }
    cached_dev = dev;
    cached_rc = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? RAPID_OK : RAPID_ERR_ARCH;
    if (cached_rc == RAPID_OK) {
        set_cu_count(prop.multiProcessorCount);
        g_probe_cus = prop.multiProcessorCount;
    }
    if (cached_rc != RAPID_OK) set_error("device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);
    return cached_rc;
}

int check_launch(const char* what) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: %s", what, hipGetErrorString(e));
        return RAPID_ERR_HIP;
    }
    return RAPID_OK;
}

template <class T>
T* at(void* ws, size_t off) { return (T*)((char*)ws + off); }

struct FwdIo {
    const void* hidden; const void* W; const int32_t* tokens; const uint8_t* mask;
    int w_layout; float temperature;
    float* logp_out; float* lse_out; int32_t* dev_status;
    bf16_t* zc = nullptr;   // if set: [row_cap, ldv], the forward also stores the ratios p_v / p_y there
    int64_t row_cap = INT64_MAX;   // compact rows the caller's buffers hold (the cache may be sized for fewer than N*T)
    const float* ref_logp = nullptr;    // with zc: the behaviour log-probs, for the reference of the stored values
    const void* rms_weight = nullptr;   // if set (bf16 only): hidden is normalised while it is packed
    float rms_eps = 0.f;
    // if idle.idle is set (backward call, bf16): the rows of the generations it marks come behind the others and
    // the chunk table's one entry says where those end
    IdleArgs idle;
    const int32_t* group_ids = nullptr;
};

// packs W as [Vpad, ldk] (the operand of the logits kernels)
void pack_w_for_logits(const Plan& p, void* ws, const void* W, int w_layout, hipStream_t st) {
    bf16_t* Wvd = at<bf16_t>(ws, p.Wvd);
    if (w_layout == RAPID_W_VD)
        launch_copy_pad_bf16((const bf16_t*)W, p.d, nullptr, Wvd, p.ldk, p.V, p.d, p.Vpad, p.dpad, nullptr, 0, st);
    else
        launch_transpose_pad_bf16((const bf16_t*)W, p.V, Wvd, p.ldk, p.d, p.V, p.dpad, p.Vpad, nullptr, 0, st);
    if (p.two_wg) launch_block_w32(Wvd, p.ldk, at<bf16_t>(ws, p.Wvd32), p.Vpad, p.dpad, st);
}

// bf16 forward over the compact rows [base, base + rows) (rows a multiple of 256; `counts` holds the end of the
// valid rows among them): token ids, packed hidden rows, sampled-token logits, streaming log-softmax, log-probs.
// Leaves tokc, seqc, zy, lse_c (and Hc) of those rows in the workspace for the backward.  Wvd is packed already.
void forward_rows_bf16(const Plan& p, void* ws, const FwdIo& io, const int32_t* counts, int64_t base, int64_t rows,
                       hipStream_t st) {
    int32_t* row_index = at<int32_t>(ws, p.row_index);
    int32_t* tokc = at<int32_t>(ws, p.tokc);
    bf16_t* Hc = at<bf16_t>(ws, p.Hc);
    const float inv_temp = 1.0f / io.temperature;
    {
        Span sp(ST_COMPACT, st);
        launch_gather_tokens(io.tokens, row_index, counts, base, rows, p.T, p.V, tokc, at<int32_t>(ws, p.seqc),
                             io.dev_status, st);
    }
    {
        Span sp(ST_PACK, st);
        if (io.rms_weight)
            launch_rmsnorm_pad_bf16((const bf16_t*)io.hidden, p.d, row_index, (const bf16_t*)io.rms_weight, io.rms_eps,
                                    Hc, p.ldk, base, rows, p.dpadR, counts, at<float>(ws, p.inv_rms), st);
        else
            launch_copy_pad_bf16((const bf16_t*)io.hidden, p.d, row_index, Hc + base * p.ldk, p.ldk, rows, p.d, rows,
                                 p.dpadR, counts, base, st);
    }
    FwdArgs a;
    a.Wvd = at<bf16_t>(ws, p.Wvd); a.Hc = Hc; a.dpad = p.dpad; a.ldk = p.ldk;
    a.tilesV = (int)(p.Vpad / 256); a.tilesM = (int)(rows / 256);
    a.V = p.V; a.inv_temp = inv_temp; a.tokc = tokc; a.counts = counts;
    a.part_max = at<float>(ws, p.part_max); a.part_sum = at<float>(ws, p.part_sum);
    a.ld_part = p.ld_part; a.zy = at<float>(ws, p.zy); a.gi = g_gi_fwd;
    a.zc = io.zc; a.ldz = p.ldv; a.dev_status = io.dev_status;
    a.refz = at<float>(ws, p.refz); a.ref_logp = io.ref_logp; a.row_index = row_index;
    a.part_row0 = base; a.zc_row0 = base;
    a.WvdB = p.two_wg ? at<bf16_t>(ws, p.Wvd32) : nullptr;
    a.k32_mode = g_fwd_two_wg.load();
    {   // the sampled tokens' logits first: a storing forward uses them as its per-row reference
        Span sp(ST_MERGE, st);
        launch_token_logit(a, base, rows, st);
    }
    // The forward runs in blocks of token rows, all vocabulary tiles per block, so that a block's
    // hidden rows stay in the memory-side cache while every XCD sweeps its share of W over them
    // (one launch over all rows re-reads the hidden rows from HBM once per group of W panels).
    const int64_t block_rows = (int64_t)g_fwd_block_tiles.load() * 256;
    for (int64_t r0 = 0; r0 < rows; r0 += block_rows) {
        const int64_t nrows = (rows - r0) < block_rows ? (rows - r0) : block_rows;
        a.row0 = base + r0;
        a.tilesM = (int)(nrows / 256);
        Span sp(ST_FWD_LSE, st);
        launch_fwd_lse(a, st);
    }
    {
        Span sp(ST_MERGE, st);
        launch_merge_lse(a.part_max, a.part_sum, p.P, a.ld_part, a.zy, row_index, counts, base, rows,
                         at<float>(ws, p.lse_c), io.logp_out, io.lse_out, st);
    }
}

// compaction, operand packing and the streaming log-softmax forward over the whole batch as one region;
// leaves lse_c, tokc, seqc, row_index, counts (and for bf16 Hc, Wvd) in the workspace for the backward
void run_forward(const Plan& p, void* ws, const FwdIo& io, hipStream_t st) {
    int32_t* counts = at<int32_t>(ws, p.counts);
    int32_t* row_index = at<int32_t>(ws, p.row_index);
    int32_t* tokc = at<int32_t>(ws, p.tokc);
    int32_t* seqc = at<int32_t>(ws, p.seqc);
    float* lse_c = at<float>(ws, p.lse_c);
    const float inv_temp = 1.0f / io.temperature;
    {
        Span sp(ST_COMPACT, st);
        if (io.idle.idle)
            launch_compaction_chunked(io.mask, io.group_ids, p.N, p.T, p.K, io.row_cap < p.Mmax_pad ? io.row_cap : p.Mmax_pad, 1,
                                      at<int32_t>(ws, p.seq_len), at<int32_t>(ws, p.cu), at<int32_t>(ws, p.tab),
                                      at<int32_t>(ws, p.gen_row0), at<int32_t>(ws, p.gen_chunk), at<int32_t>(ws, p.gseen),
                                      row_index, counts, io.dev_status, io.idle, st);
        else
            launch_compaction(io.mask, p.N, p.T, at<int32_t>(ws, p.seq_len), at<int32_t>(ws, p.cu), row_index, counts,
                              io.row_cap, io.dev_status, st);
        launch_fill_f32(io.logp_out, p.Mmax, 0.f, st);
        if (io.lse_out) launch_fill_f32(io.lse_out, p.Mmax, 0.f, st);
    }
    if (p.dtype == RAPID_DTYPE_BF16) {
        {
            Span sp(ST_PACK, st);
            pack_w_for_logits(p, ws, io.W, io.w_layout, st);
        }
        forward_rows_bf16(p, ws, io, counts, 0, p.Mmax_pad, st);
    } else {
        {
            Span sp(ST_COMPACT, st);
            launch_gather_tokens(io.tokens, row_index, counts, 0, p.Mmax_pad, p.T, p.V, tokc, seqc, io.dev_status, st);
        }
        float* z = at<float>(ws, p.chunk0);
        Span sp(ST_F32, st);
        for (int64_t m0 = 0; m0 < p.Mmax; m0 += p.Mc) {
            const int64_t rows = (p.Mmax - m0) < p.Mc ? (p.Mmax - m0) : p.Mc;
            F32Gemm g;
            memset(&g, 0, sizeof(g));
            g.A = (const float*)io.hidden; g.sa_i = p.d; g.sa_k = 1; g.a_imap = row_index;
            g.B = (const float*)io.W;
            if (io.w_layout == RAPID_W_DV) { g.sb_k = p.V; g.sb_j = 1; } else { g.sb_k = 1; g.sb_j = p.d; }
            g.C = z; g.sc_i = p.V; g.sc_j = 1;
            g.I = rows; g.J = p.V; g.Kd = p.d; g.beta = 0; g.counts = counts; g.i0 = m0; g.limit_k = 0;
            g.alpha = inv_temp;
            launch_f32_gemm(g, st);
            launch_f32_row_lse(z, p.V, rows, m0, tokc, row_index, counts, lse_c, io.logp_out, io.lse_out, st);
        }
    }
}

int validate_common(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask, int64_t d,
                    int dtype, int w_layout, float temperature, void* workspace) {
    if (!hidden || !W || !tokens || !mask) {
        set_error("hidden, W, tokens and mask must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (w_layout != RAPID_W_DV && w_layout != RAPID_W_VD) {
        set_error("unknown w_layout %d", w_layout);
        return RAPID_ERR_DTYPE;
    }
    if (!(temperature > 0.f) || !std::isfinite(temperature)) {
        set_error("temperature must be finite and > 0");
        return RAPID_ERR_SHAPE;
    }
    if (dtype == RAPID_DTYPE_BF16 && d % 8 != 0) {
        set_error("bf16 needs d %% 8 == 0 (got d = %lld)", (long long)d);
        return RAPID_ERR_SHAPE;
    }
    if (((uintptr_t)hidden | (uintptr_t)W) % 16 != 0) {
        set_error("hidden and W must be 16-byte aligned");
        return RAPID_ERR_SHAPE;
    }
    if (!workspace || ((uintptr_t)workspace) % 256 != 0) {
        set_error("workspace must be non-NULL and 256-byte aligned");
        return RAPID_ERR_WORKSPACE;
    }
    return RAPID_OK;
}

int validate_rms(const void* rms_weight, float rms_eps, int dtype) {
    if (!rms_weight) return RAPID_OK;
    if (dtype != RAPID_DTYPE_BF16) {
        set_error("rms_weight needs bf16 inputs");
        return RAPID_ERR_DTYPE;
    }
    if (((uintptr_t)rms_weight) % 16 != 0 || !(rms_eps >= 0.f) || !std::isfinite(rms_eps)) {
        set_error("rms_weight must be 16-byte aligned and rms_eps finite and >= 0");
        return RAPID_ERR_SHAPE;
    }
    return RAPID_OK;
}

int logprob_fwd(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask, int64_t N, int64_t T,
                int64_t d, int64_t V, int dtype, int w_layout, float temperature, const void* rms_weight,
                float rms_eps, float* logp_out, float* lse_out, int32_t* dev_status, void* workspace,
                size_t workspace_bytes, void* stream) {
    Plan p;
    if (!make_plan(p, RAPID_OP_LOGPROB_FWD, N, T, d, V, 1, dtype)) {
        set_error("bad shape/dtype N=%lld T=%lld d=%lld V=%lld dtype=%d", (long long)N, (long long)T, (long long)d,
                  (long long)V, dtype);
        return (dtype != RAPID_DTYPE_F32 && dtype != RAPID_DTYPE_BF16) ? RAPID_ERR_DTYPE : RAPID_ERR_SHAPE;
    }
    int rc = validate_common(hidden, W, tokens, mask, d, dtype, w_layout, temperature, workspace);
    if (rc) return rc;
    rc = validate_rms(rms_weight, rms_eps, dtype);
    if (rc) return rc;
    if (!logp_out) {
        set_error("logp_out must not be NULL");
        return RAPID_ERR_NULL;
    }
    const int64_t Mc = fit_chunk(p, workspace_bytes);
    if (Mc < ROW_TILE) {
        set_error("workspace of %zu bytes is below the minimum %zu", workspace_bytes,
                  rapid_workspace_min_bytes(RAPID_OP_LOGPROB_FWD, N, T, d, V, 1, dtype));
        return RAPID_ERR_WORKSPACE;
    }
    size_chunks(p, Mc < recommended_chunk(p) ? Mc : recommended_chunk(p));
    rc = check_arch();
    if (rc) return rc;
    FwdIo io{hidden, W, tokens, mask, w_layout, temperature, logp_out, lse_out, dev_status};
    io.rms_weight = rms_weight;
    io.rms_eps = rms_eps;
    run_forward(p, workspace, io, (hipStream_t)stream);
    return check_launch("rapid_logprob_fwd");
}

}  // namespace
}  // namespace rapid

using namespace rapid;

extern "C" {

int rapid_version(void) { return 7; }

const char* rapid_last_error(void) { return g_err; }

void rapid_iw_pg_default_opts(rapid_iw_pg_opts* o) {
    if (!o) return;
    memset(o, 0, sizeof(*o));
    o->eta = 2.0f;
    o->coef_mode = 0;
    o->baseline_mode = 0;
    o->loss_scale = 1.0f;
    o->temperature = 1.0f;
    o->w_layout = RAPID_W_DV;
    o->dw_dtype = RAPID_DTYPE_F32;
    o->accumulate_dw = 0;
    o->normalized_grads = 0;
    o->logits_cache = 0;
    o->ratio_level = 0;
    o->max_tokens = 0;
    o->rms_weight = nullptr;
    o->drms_weight_out = nullptr;
    o->rms_eps = 1e-6f;
    o->coef_override = nullptr;
}

int rapid_set_tuning(int key, int value) {
    if (key >= 10 && key <= 12 && value >= 0 && value <= 1024) {
        (key == 10 ? g_gi_fwd : key == 11 ? g_gi_dh : g_gi_dw).store((key != 11 && value == 0) ? 1 : value);
        return RAPID_OK;
    }
    if (key == 13 && value >= 1 && value <= (1 << 20)) {
        g_fwd_block_tiles = value;
        return RAPID_OK;
    }
    if (key == 15 && value >= 0 && value <= (1 << 20)) {
        g_cached_step_tiles = value;
        return RAPID_OK;
    }
    if (key == 16 && value >= 0 && value <= 4096 && (value & (value - 1)) == 0) {
        g_pace_every = value;
        return RAPID_OK;
    }
    if (key == 14 && (value == 0 || value == 1)) {
        g_blocked_wdv = value;
        return RAPID_OK;
    }
    if (key == 17 && (value == 0 || value == 1)) {
        g_dh_split = value;
        return RAPID_OK;
    }
    if (key == 22 && (value == 0 || value == 1)) {
        set_dw_deep(value);
        return RAPID_OK;
    }
    if (key == 21 && value >= 0 && value <= 3) {
        g_fwd_two_wg = value;
        return RAPID_OK;
    }
    if (key == 20 && value >= 0) {
        g_cached_dw_step_tiles = value;
        return RAPID_OK;
    }
    if (key == 19 && (value == 0 || value == 1)) {
        g_skip_idle = value;
        return RAPID_OK;
    }
    if (key == 18 && value >= ROW_TILE && value % ROW_TILE == 0) {
        g_cached_rcap = value;
        return RAPID_OK;
    }
    if (key == 2 && (value == 0 || value == 4 || value == 8 || value == 16)) {
        set_waves_per_workgroup(value);
        return RAPID_OK;
    }
    if (key == 1 && (value == 0 || value == 1)) {
        g_prof.on = value != 0;
        g_prof.used = 0;
        return RAPID_OK;
    }
    set_error("unknown tuning key/value %d/%d", key, value);
    return RAPID_ERR_DTYPE;
}

int rapid_sgd_step(float* master, const float* grad, int64_t n, float lr, void* w_out, int dtype, void* stream) {
    if (!master || !grad) {
        set_error("master and grad must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (n <= 0 || !std::isfinite(lr)) {
        set_error("n must be > 0 and lr finite");
        return RAPID_ERR_SHAPE;
    }
    if (dtype != RAPID_DTYPE_F32 && dtype != RAPID_DTYPE_BF16) {
        set_error("unknown dtype %d", dtype);
        return RAPID_ERR_DTYPE;
    }
    int rc = check_arch();
    if (rc) return rc;
    launch_sgd_step(master, grad, n, lr, w_out, dtype, (hipStream_t)stream);
    return check_launch("rapid_sgd_step");
}

int rapid_adamw_step(float* master, const float* grad, float* exp_avg, float* exp_avg_sq, int64_t n, float lr,
                     float beta1, float beta2, float eps, float weight_decay, int64_t step, void* w_out, int dtype,
                     void* stream) {
    if (!master || !grad || !exp_avg || !exp_avg_sq) {
        set_error("master, grad, exp_avg and exp_avg_sq must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (n <= 0 || step < 1 || !std::isfinite(lr) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) ||
        !(eps >= 0.f) || !std::isfinite(eps) || !std::isfinite(weight_decay)) {
        set_error("n > 0, step >= 1, lr finite, betas in [0, 1), eps >= 0 and weight_decay finite are required");
        return RAPID_ERR_SHAPE;
    }
    if (dtype != RAPID_DTYPE_F32 && dtype != RAPID_DTYPE_BF16) {
        set_error("unknown dtype %d", dtype);
        return RAPID_ERR_DTYPE;
    }
    int rc = check_arch();
    if (rc) return rc;
    launch_adamw_step(master, grad, exp_avg, exp_avg_sq, n, lr, beta1, beta2, eps, weight_decay, step, w_out, dtype,
                      (hipStream_t)stream);
    return check_launch("rapid_adamw_step");
}

int rapid_seq_logratio(const float* logp_cur, const float* logp_behav, const uint8_t* mask, int64_t N, int64_t T,
                       float* tok_logratio_out, float* seq_logratio_out, int32_t* dev_status, void* stream) {
    if (!logp_cur || !logp_behav || !mask || !seq_logratio_out) {
        set_error("logp_cur, logp_behav, mask and seq_logratio_out must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (N <= 0 || T <= 0 || N * T > (int64_t)2000000000) {
        set_error("bad shape N=%lld T=%lld", (long long)N, (long long)T);
        return RAPID_ERR_SHAPE;
    }
    int rc = check_arch();
    if (rc) return rc;
    launch_seq_logratio(logp_cur, logp_behav, mask, N, T, tok_logratio_out, nullptr, seq_logratio_out, 2.f, 0, nullptr,
                        nullptr, nullptr, dev_status, (hipStream_t)stream);
    return check_launch("rapid_seq_logratio");
}

int rapid_mfma_probe(int random_operands, int iters, double* tflops_out, double* ms_out, void* stream) {
    if (iters < 1 || iters > 10000000) {
        set_error("iters must be in 1 .. 10^7");
        return RAPID_ERR_SHAPE;
    }
    int rc = check_arch();
    if (rc) return rc;
    rc = run_mfma_probe(random_operands != 0, iters, g_probe_cus, tflops_out, ms_out, (hipStream_t)stream);
    if (rc) {
        set_error("rapid_mfma_probe: HIP event or launch failure");
        return rc;
    }
    return check_launch("rapid_mfma_probe");
}

int rapid_profile_read(double* ms_by_stage, int64_t* spans_by_stage, int n_stages) {
    if (!ms_by_stage || !spans_by_stage || n_stages < ST_COUNT) {
        set_error("rapid_profile_read needs two arrays of at least %d entries", (int)ST_COUNT);
        return RAPID_ERR_NULL;
    }
    for (int i = 0; i < n_stages; ++i) { ms_by_stage[i] = 0.0; spans_by_stage[i] = 0; }
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess) {
            set_error("rapid_profile_read: event query failed");
            g_prof.used = 0;
            return RAPID_ERR_HIP;
        }
        ms_by_stage[g_prof.stage[i]] += ms;
        spans_by_stage[g_prof.stage[i]] += 1;
    }
    g_prof.used = 0;
    return RAPID_OK;
}

// cached backward, cache large enough for every token the batch may hold: one chunk
size_t rapid_workspace_bytes_max_tokens(int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype,
                                        int64_t max_tokens) {
    if (op != RAPID_OP_IW_PG_FWD_BWD_CACHED) return rapid_workspace_bytes(op, N, T, d, V, K, dtype);
    Plan p;
    if (max_tokens < 0 || dtype != RAPID_DTYPE_BF16 || !make_plan(p, RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, dtype))
        return 0;
    const int64_t rows = cache_rows(p, max_tokens);
    return cached_total(N, T, d, V, K, rows, rows);
}

int64_t rapid_logits_cache_rows(int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int64_t max_tokens, size_t workspace_bytes) {
    Plan p;
    if (max_tokens < 0 || !make_plan(p, RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, RAPID_DTYPE_BF16)) return 0;
    return choose_cache(N, T, d, V, K, cache_rows(p, max_tokens), workspace_bytes, &p);
}

size_t rapid_workspace_bytes(int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype) {
    if (op == RAPID_OP_GROUP_ADVANTAGE) return 0;
    Plan p;
    if (op == RAPID_OP_IW_PG_FWD_BWD_CACHED) {   // a cache of the recommended number of rows, or of all rows if those are fewer
        if (dtype != RAPID_DTYPE_BF16 || !make_plan(p, RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, dtype)) return 0;
        return cached_total(N, T, d, V, K, p.Mmax_pad, g_cached_rcap.load());
    }
    if (op != RAPID_OP_LOGPROB_FWD && op != RAPID_OP_IW_PG_FWD_BWD) return 0;
    if (!make_plan(p, op, N, T, d, V, K, dtype)) return 0;
    size_chunks(p, recommended_chunk(p));
    return p.total + 1024;
}

size_t rapid_workspace_min_bytes(int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype) {
    if (op == RAPID_OP_GROUP_ADVANTAGE) return 0;
    Plan p;
    if (op == RAPID_OP_IW_PG_FWD_BWD_CACHED) {   // a cache of one row tile (every group must fit into it)
        if (dtype != RAPID_DTYPE_BF16 || !make_plan(p, RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, dtype)) return 0;
        return cached_total(N, T, d, V, K, p.Mmax_pad, ROW_TILE);
    }
    if (op != RAPID_OP_LOGPROB_FWD && op != RAPID_OP_IW_PG_FWD_BWD) return 0;
    if (!make_plan(p, op, N, T, d, V, K, dtype)) return 0;
    size_chunks(p, ROW_TILE);
    return p.total + 1024;
}

int rapid_compaction(const uint8_t* mask, int64_t N, int64_t T, int32_t* seq_len_out, int32_t* cu_seqlen_out,
                     int32_t* row_index_out, void* stream) {
    if (!mask || !seq_len_out || !cu_seqlen_out) {
        set_error("mask, seq_len_out and cu_seqlen_out must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (N <= 0 || T <= 0 || N * T > (int64_t)2000000000) {
        set_error("bad shape N=%lld T=%lld", (long long)N, (long long)T);
        return RAPID_ERR_SHAPE;
    }
    int rc = check_arch();
    if (rc) return rc;
    launch_compaction(mask, N, T, seq_len_out, cu_seqlen_out, row_index_out, nullptr, INT64_MAX, nullptr,
                      (hipStream_t)stream);
    return check_launch("rapid_compaction");
}

int rapid_logprob_fwd(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask, int64_t N,
                      int64_t T, int64_t d, int64_t V, int dtype, int w_layout, float temperature, float* logp_out,
                      float* lse_out, int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream) {
    return logprob_fwd(hidden, W, tokens, mask, N, T, d, V, dtype, w_layout, temperature, nullptr, 0.f, logp_out,
                       lse_out, dev_status, workspace, workspace_bytes, stream);
}

int rapid_logprob_fwd_static(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask, int64_t N,
                             int64_t T, int64_t d, int64_t V, int dtype, int w_layout, float temperature,
                             float* logp_out, float* lse_out, int32_t* dev_status, void* stream) {
    const size_t need = rapid_workspace_min_bytes(RAPID_OP_LOGPROB_FWD, N, T, d, V, 1, dtype);
    if (need == 0) {
        set_error("bad shape/dtype N=%lld T=%lld d=%lld V=%lld dtype=%d", (long long)N, (long long)T, (long long)d,
                  (long long)V, dtype);
        return (dtype != RAPID_DTYPE_F32 && dtype != RAPID_DTYPE_BF16) ? RAPID_ERR_DTYPE : RAPID_ERR_SHAPE;
    }
    if (need > RAPID_STATIC_SCRATCH_BYTES) {
        set_error("rapid_logprob_fwd_static: this shape needs %zu bytes of scratch, the static scratch holds %zu; "
                  "use rapid_logprob_fwd with a workspace", need, (size_t)RAPID_STATIC_SCRATCH_BYTES);
        return RAPID_ERR_WORKSPACE;
    }
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc) return rc;
    return logprob_fwd(hidden, W, tokens, mask, N, T, d, V, dtype, w_layout, temperature, nullptr, 0.f, logp_out,
                       lse_out, dev_status, ptr, RAPID_STATIC_SCRATCH_BYTES, stream);
}

int rapid_logprob_fwd_rmsnorm(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask, int64_t N,
                              int64_t T, int64_t d, int64_t V, int dtype, int w_layout, float temperature,
                              const void* rms_weight, float rms_eps, float* logp_out, float* lse_out,
                              int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream) {
    if (!rms_weight) {
        set_error("rms_weight must not be NULL");
        return RAPID_ERR_NULL;
    }
    return logprob_fwd(hidden, W, tokens, mask, N, T, d, V, dtype, w_layout, temperature, rms_weight, rms_eps,
                       logp_out, lse_out, dev_status, workspace, workspace_bytes, stream);
}

int rapid_group_advantage(const float* rewards, const int32_t* group_ids, const float* seq_logratio, int64_t N,
                          int64_t K, float eta, int baseline_mode, float* adv_out, float* weight_out,
                          float* group_mean_out, float* group_std_out, int32_t* group_size_out, int32_t* dev_status,
                          void* stream) {
    if (!rewards || !group_ids || !adv_out) {
        set_error("rewards, group_ids and adv_out must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (N <= 0 || K <= 0 || N > (int64_t)2000000000 || K > (int64_t)2000000000) {
        set_error("bad shape N=%lld K=%lld", (long long)N, (long long)K);
        return RAPID_ERR_SHAPE;
    }
    if (baseline_mode < 0 || baseline_mode > 2) {
        set_error("unknown baseline_mode %d", baseline_mode);
        return RAPID_ERR_DTYPE;
    }
    if (!(eta > 0.f)) {
        set_error("eta must be > 0 (inf allowed)");
        return RAPID_ERR_SHAPE;
    }
    int rc = check_arch();
    if (rc) return rc;
    launch_group_advantage(rewards, group_ids, seq_logratio, nullptr, N, K, eta, baseline_mode, adv_out, nullptr, weight_out,
                           group_mean_out, group_std_out, group_size_out, nullptr, dev_status, (hipStream_t)stream);
    return check_launch("rapid_group_advantage");
}

}  // extern "C"

// The clipped token-level surrogate of the baselines' loss steps, when the fused path runs for them: the
// estimator stage differs (normalised advantages, per-token coefficients), everything else is shared.
struct ClipSpec {
    rapid_clip_pg_opts o;
    const float* logp_ref;
    rapid_clip_pg_diag* diag;
};

static int fused_call(const char* name, const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                      const float* logp_behav, const float* rewards, const int32_t* group_ids, int64_t N,
                      int64_t T, int64_t d, int64_t V, int64_t K, int dtype, const rapid_iw_pg_opts& o,
                      float* loss_out, void* dhidden_out, void* dW_out, float* logp_cur_out,
                      float* tok_logratio_out, float* seq_logratio_out, float* adv_out,
                      rapid_iw_pg_diag* diag_out, int32_t* dev_status, void* workspace,
                      size_t workspace_bytes, void* stream, const ClipSpec* clip) {
    Plan p;
    if (!make_plan(p, RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, dtype)) {
        set_error("bad shape/dtype N=%lld T=%lld d=%lld V=%lld K=%lld dtype=%d", (long long)N, (long long)T,
                  (long long)d, (long long)V, (long long)K, dtype);
        return (dtype != RAPID_DTYPE_F32 && dtype != RAPID_DTYPE_BF16) ? RAPID_ERR_DTYPE : RAPID_ERR_SHAPE;
    }
    int rc = validate_common(hidden, W, tokens, mask, d, dtype, o.w_layout, o.temperature, workspace);
    if (rc) return rc;
    if (!rewards || !group_ids || !loss_out || !dhidden_out || !dW_out) {
        set_error("rewards, group_ids, loss_out, dhidden_out and dW_out must not be NULL");
        return RAPID_ERR_NULL;
    }
    if (o.coef_mode < 0 || o.coef_mode > 1 || o.baseline_mode < 0 || o.baseline_mode > 2 || o.ratio_level < 0 ||
        o.ratio_level > 1 || (o.dw_dtype != RAPID_DTYPE_F32 && o.dw_dtype != RAPID_DTYPE_BF16)) {
        set_error("unknown coef_mode / baseline_mode / ratio_level / dw_dtype");
        return RAPID_ERR_DTYPE;
    }
    if (!(o.eta > 0.f) || !(o.loss_scale > 0.f) || !std::isfinite(o.loss_scale)) {
        set_error("eta must be > 0 (inf allowed) and loss_scale finite and > 0");
        return RAPID_ERR_SHAPE;
    }
    if (o.accumulate_dw && o.dw_dtype != RAPID_DTYPE_F32) {
        set_error("accumulate_dw needs an fp32 dW");
        return RAPID_ERR_DTYPE;
    }
    if (o.logits_cache != 0 && (o.logits_cache != 1 || dtype != RAPID_DTYPE_BF16)) {
        set_error("logits_cache must be 0 or 1, and 1 needs bf16 inputs");
        return RAPID_ERR_DTYPE;
    }
    if (((uintptr_t)dhidden_out | (uintptr_t)dW_out) % 16 != 0) {
        set_error("dhidden_out and dW_out must be 16-byte aligned");
        return RAPID_ERR_SHAPE;
    }
    const bool cached = o.logits_cache == 1;
    if (o.max_tokens < 0) {
        set_error("max_tokens must be >= 0");
        return RAPID_ERR_SHAPE;
    }
    rc = validate_rms(o.rms_weight, o.rms_eps, dtype);
    if (rc) return rc;
    if (cached) {
        // The cache holds every token if the workspace allows (one chunk: groups may lie anywhere in the
        // batch); otherwise as many rows as fit, and the batch is worked through in chunks of whole groups.
        if (choose_cache(N, T, d, V, K, cache_rows(p, o.max_tokens), workspace_bytes, &p) == 0) {
            set_error("workspace of %zu bytes is below the %zu the logits cache needs at least", workspace_bytes,
                      rapid_workspace_min_bytes(RAPID_OP_IW_PG_FWD_BWD_CACHED, N, T, d, V, K, dtype));
            return RAPID_ERR_WORKSPACE;
        }
    } else {
        const int64_t Mfit = fit_chunk(p, workspace_bytes);
        if (Mfit < ROW_TILE) {
            set_error("workspace of %zu bytes is below the minimum %zu", workspace_bytes,
                      rapid_workspace_min_bytes(RAPID_OP_IW_PG_FWD_BWD, N, T, d, V, K, dtype));
            return RAPID_ERR_WORKSPACE;
        }
        // the fp32 path launches one block row per 16 chunk rows along the second grid dimension: its chunk
        // stays at the recommended size however large the workspace is
        size_chunks(p, (dtype == RAPID_DTYPE_F32 && Mfit > recommended_chunk(p)) ? recommended_chunk(p) : Mfit);
    }
    rc = check_arch();
    if (rc) return rc;

    hipStream_t st = (hipStream_t)stream;
    void* ws = workspace;
    int32_t* counts = at<int32_t>(ws, p.counts);
    int32_t* row_index = at<int32_t>(ws, p.row_index);
    int32_t* tokc = at<int32_t>(ws, p.tokc);
    int32_t* seqc = at<int32_t>(ws, p.seqc);
    float* lse_c = at<float>(ws, p.lse_c);
    float* logp_cur = logp_cur_out ? logp_cur_out : at<float>(ws, p.logp_tmp);
    double* s64 = at<double>(ws, p.s64);
    float* s32 = seq_logratio_out ? seq_logratio_out : at<float>(ws, p.s32);
    float* adv = adv_out ? adv_out : at<float>(ws, p.adv);
    double* adv64 = at<double>(ws, p.adv64);
    float* g = at<float>(ws, p.g);
    float* rowg = at<float>(ws, p.rowg);
    const float inv_temp = 1.0f / o.temperature;
    const int elem = dtype == RAPID_DTYPE_BF16 ? 2 : 4;
    // token-level outer weight: per generation the sum and the log-maximum of its tokens' ratios
    const bool per_token = o.ratio_level == 1 && !o.coef_override;
    double* tsum = per_token ? at<double>(ws, p.tsum) : nullptr;
    double* tmax = per_token ? at<double>(ws, p.tmax) : nullptr;
    CoefArgs ca;
    memset(&ca, 0, sizeof(ca));
    ca.s64 = s64; ca.adv = adv; ca.adv64 = adv64; ca.coef_override = o.coef_override; ca.N = N; ca.eta = o.eta;
    ca.coef_mode = o.coef_mode; ca.loss_scale = o.loss_scale; ca.normalized = o.normalized_grads;
    ca.tsum = tsum; ca.tmax = tmax; ca.counts = counts; ca.g = g; ca.g64 = at<double>(ws, p.g64);
    ca.loss_out = loss_out; ca.diag = diag_out; ca.write_g = 1;

    ClipArgs cl;
    memset(&cl, 0, sizeof(cl));
    if (clip) {
        cl.logp_cur = logp_cur; cl.logp_old = logp_behav; cl.logp_ref = clip->o.kl_beta != 0.f ? clip->logp_ref : nullptr;
        cl.mask = mask; cl.adv64 = adv64; cl.seq_len = at<int32_t>(ws, p.seq_len); cl.counts = counts; cl.N = N; cl.T = T;
        cl.eps_low = clip->o.eps_low; cl.eps_high = clip->o.eps_high; cl.kl_beta = clip->o.kl_beta;
        cl.loss_scale = clip->o.loss_scale; cl.norm_mode = clip->o.norm_mode;
    }

    // where each group lies in the batch: groups that are one run are reduced over that run alone
    int32_t* gruns = at<int32_t>(ws, p.gruns);
    launch_group_runs(group_ids, N, K, gruns, st);

    FwdIo io{hidden, W, tokens, mask, o.w_layout, o.temperature, logp_cur, nullptr, dev_status};
    io.rms_weight = o.rms_weight;
    io.rms_eps = o.rms_eps;

    if (cached) {
        // ---- cached backward: chunk after chunk of whole groups; forward with store, estimator, dHidden, dW
        bf16_t* Hc = at<bf16_t>(ws, p.Hc);
        bf16_t* cache = at<bf16_t>(ws, p.chunk0);
        int32_t* tab = at<int32_t>(ws, p.tab);
        int32_t* gen_chunk = at<int32_t>(ws, p.gen_chunk);
        double* lam_state = at<double>(ws, p.lam_state);
        double* lam_chunk = at<double>(ws, p.lam_chunk);
        float* beta_scale = at<float>(ws, p.beta_scale);
        // a normalised gradient that is added to the caller's dW goes through a buffer of its own: the
        // running rescaling of the sum must not touch what the caller had in dW
        const bool dw_staged = o.dw_dtype == RAPID_DTYPE_BF16 || (o.accumulate_dw && o.normalized_grads && p.Cmax > 1);
        float* dW32 = dw_staged ? at<float>(ws, p.dw32) : (float*)dW_out;
        const bool dw_adds_to_caller = o.accumulate_dw && !dw_staged;
        io.zc = cache;
        io.ref_logp = logp_behav;
        // Generations whose coefficient is zero before any log-prob is known (a group whose rewards are all 0, or a
        // zero override) come last inside their chunk, and dHidden and dW stop in front of them.  With the
        // baselines' KL term every token carries gradient: nothing is idle then.
        IdleArgs idle_args;
        if (g_skip_idle.load() && !(clip && clip->o.kl_beta != 0.f)) {
            idle_args.rewards = rewards; idle_args.coef_override = clip ? nullptr : o.coef_override;
            idle_args.idle = at<int32_t>(ws, p.idle); idle_args.len_live = at<int32_t>(ws, p.len_live);
            idle_args.cu_live = at<int32_t>(ws, p.cu_live); idle_args.live_group = at<int32_t>(ws, p.live_group);
        }
        {
            Span sp(ST_COMPACT, st);
            launch_compaction_chunked(mask, group_ids, N, T, K, p.Rcap, p.Cmax, at<int32_t>(ws, p.seq_len),
                                      at<int32_t>(ws, p.cu), tab, at<int32_t>(ws, p.gen_row0), gen_chunk,
                                      at<int32_t>(ws, p.gseen), row_index, counts, dev_status, idle_args, st);
            launch_fill_f32(logp_cur, p.Mmax, 0.f, st);
            launch_fill_f64(lam_state, 1, -INFINITY, st);
        }
        const bool blocked_wdv = g_blocked_wdv.load() != 0;
        {
            Span sp(ST_PACK, st);
            pack_w_for_logits(p, ws, W, o.w_layout, st);
            bf16_t* Wdv = at<bf16_t>(ws, p.Wdv);
            if (o.w_layout == RAPID_W_DV)
                launch_copy_pad_bf16((const bf16_t*)W, p.V, nullptr, Wdv, p.ldv, p.d, p.V, p.dpadR, p.Vpad, nullptr, 0, st);
            else
                launch_transpose_pad_bf16((const bf16_t*)W, p.d, Wdv, p.ldv, p.V, p.d, p.Vpad, p.dpadR, nullptr, 0, st);
            if (blocked_wdv)
                launch_block_rows_bf16(Wdv, p.ldv, at<bf16_t>(ws, p.WdvB), p.dpadR, p.Vpad, p.dpadR % 256 == 0 ? 256 : 128, st);
        }
        {
            Span sp(ST_ZERO, st);
            launch_zero_masked_rows(dhidden_out, mask, p.Mmax, d, elem, idle_args.idle, T, st);
        }
        const int cst = g_cached_step_tiles.load();
        const int64_t cstep = cst > 0 ? ((int64_t)cst * ROW_TILE < p.Rcap ? (int64_t)cst * ROW_TILE : p.Rcap) : p.Rcap;
        const int wst = g_cached_dw_step_tiles.load();
        const int64_t wstep = wst > 0 ? ((int64_t)wst * ROW_TILE < p.Rcap ? (int64_t)wst * ROW_TILE : p.Rcap) : p.Rcap;
        const int pace_every = g_pace_every.load();
        for (int c = 0; c < p.Cmax; ++c) {
            const int64_t base = (int64_t)c * p.Rcap;
            const int32_t* cnt = tab + (int64_t)c * CH_WORDS;     // this chunk's row counters
            const int32_t* gen_range = cnt + CH_G0;
            forward_rows_bf16(p, ws, io, cnt, base, p.Rcap, st);
            if (clip) {
                Span sp(ST_ESTIMATOR, st);
                launch_group_advantage(rewards, group_ids, nullptr, nullptr, N, K, 2.f, BASELINE_NORMALIZED, adv, adv64, nullptr,
                                       nullptr, nullptr, nullptr, gen_range, dev_status, st, clip->o.adv_eps, clip->o.std_ddof, gruns);
                launch_clip_generations(cl, gen_range, at<double>(ws, p.g64), at<double>(ws, p.tsum), at<double>(ws, p.tmax),
                                        dev_status, st);
                launch_clip_rows(cl, seqc, row_index, cnt, base, p.Rcap, rowg, st);
            } else {
                Span sp(ST_ESTIMATOR, st);
                launch_seq_logratio(logp_cur, logp_behav, mask, N, T, tok_logratio_out, s64, s32, o.eta, o.coef_mode == 1,
                                    tsum, tmax, gen_range, dev_status, st);
                launch_group_advantage(rewards, group_ids, nullptr, logp_behav ? s64 : nullptr, N, K, o.eta, o.baseline_mode,
                                       adv, adv64, nullptr, nullptr, nullptr, nullptr, gen_range, dev_status, st, 0.f, 0, gruns);
                CoefArgs cc = ca;
                cc.gen_range = gen_range; cc.lam_state = lam_state; cc.lam_chunk = lam_chunk + c; cc.beta_out = beta_scale;
                launch_coefficients(cc, st);
                launch_row_coefficients(g, ca.g64, seqc, row_index, cnt, logp_cur, logp_behav, per_token, o.eta,
                                        o.coef_mode == 1, base, p.Rcap, rowg, st);
            }
            {   // row factors, the sampled tokens' elements, hidden rows scaled by the factors
                Span sp(ST_DZ, st);
                launch_cache_finish(cache, p.ldv, Hc, p.ldk, tokc, at<float>(ws, p.zy), at<float>(ws, p.refz), lse_c, rowg,
                                    inv_temp, cnt, base, p.Rcap, at<float>(ws, p.rowc), dev_status, st);
            }
            // dHidden of the chunk in pieces of cstep rows (a launch boundary keeps the XCDs' sweeps over W together), then
            // dW over all its rows at once (every dW launch re-reads and re-writes all of dW and ends in a tail: one
            // launch per chunk is 1.3 % faster than one per 65536 rows).  (Running dW on a second stream beside dHidden,
            // so that it fills the compute units a short last round of dHidden tiles leaves idle, was tried: the
            // two kernels are dispatched side by side from the start, each XCD then holds half as many workgroups
            // of either, they share fewer operand panels in its L2, and the pair takes 4 % longer.)
            for (int64_t r0 = 0; r0 < p.Rcap; r0 += cstep) {
                const int64_t rows = (p.Rcap - r0) < cstep ? (p.Rcap - r0) : cstep;
                DhArgs ha;
                ha.Wdv = at<bf16_t>(ws, p.Wdv); ha.WdvB = blocked_wdv ? at<bf16_t>(ws, p.WdvB) : nullptr; ha.dz = cache + r0 * p.ldv;
                ha.Vpad = p.Vpad; ha.ldv = p.ldv; ha.d = p.d; ha.dpadR = p.dpadR;
                ha.tilesM = (int)(rows / 256); ha.m0 = base + r0; ha.row_index = row_index; ha.counts = cnt + CH_LIVE;
                ha.rowc = at<float>(ws, p.rowc);
                ha.pace = pace_every > 0 ? at<unsigned>(ws, p.pace) : nullptr; ha.pace_every = pace_every;
                if (ha.pace) launch_fill_f32((float*)ha.pace, 64, 0.f, st);
                ha.dhidden = (bf16_t*)dhidden_out; ha.gi = g_gi_dh;
                ha.part = g_dh_split.load() ? at<float>(ws, p.dh_part) : nullptr; ha.part_bytes = dh_part_bytes();
                Span sp(ST_DH, st);
                launch_dh(ha, st);
            }
            int piece = 0;
            for (int64_t r0 = 0; r0 < p.Rcap; r0 += wstep, ++piece) {
                const int64_t rows = (p.Rcap - r0) < wstep ? (p.Rcap - r0) : wstep;
                DwArgs wa;
                wa.dz = cache + r0 * p.ldv; wa.Hc = Hc + (base + r0) * p.ldk; wa.Mc = rows; wa.ldz = p.ldv; wa.ldH = p.ldk;
                wa.d = p.d; wa.dpadR = p.dpadR; wa.V = p.V; wa.Vpad = p.Vpad; wa.m0 = base + r0; wa.counts = cnt + CH_LIVE;
                wa.dW = dW32; wa.w_layout = o.w_layout; wa.gi = g_gi_dw;
                wa.beta = (c > 0 || piece > 0 || dw_adds_to_caller) ? 1 : 0;
                // the sum over the earlier chunks is brought to this chunk's scale, once, by its first piece
                wa.beta_scale = (c > 0 && piece == 0 && o.normalized_grads && !dw_adds_to_caller) ? beta_scale : nullptr;
                Span sp(ST_DW, st);
                launch_dw(wa, st);
            }
        }
        {   // loss and diagnostics of the whole batch (every generation's ratio and advantage is known now)
            Span sp(ST_ESTIMATOR, st);
            if (clip) {
                launch_clip_finish(at<double>(ws, p.g64), at<double>(ws, p.tsum), at<double>(ws, p.tmax), N, counts, loss_out,
                                   clip->diag, st);
            } else {
                CoefArgs cf = ca;
                cf.write_g = 0;
                launch_coefficients(cf, st);
            }
        }
        if (o.normalized_grads && p.Cmax > 1) {   // rows of earlier chunks: from their chunk's scale to the final one
            Span sp(ST_ZERO, st);
            launch_rescale_rows(dhidden_out, mask, N, T, d, gen_chunk, lam_chunk, lam_state, st);
        }
        if (o.rms_weight) {   // dhidden holds dL/dh of the normalised state: on to dL/dweight and dL/dx
            Span sp(ST_ZERO, st);
            float* part = o.drms_weight_out ? at<float>(ws, p.rms_part) : nullptr;
            if (part) launch_fill_f32(part, p.rms_blocks * d, 0.f, st);
            const int64_t blocks_per_region = rmsnorm_dweight_blocks(p.Rcap);
            for (int c = 0; c < p.Cmax; ++c)
                launch_rmsnorm_backward((const bf16_t*)hidden, (bf16_t*)dhidden_out, d, (const bf16_t*)o.rms_weight, row_index,
                                        tab + (int64_t)c * CH_WORDS, at<float>(ws, p.inv_rms), (int64_t)c * p.Rcap, p.Rcap,
                                        part ? part + (int64_t)c * blocks_per_region * d : nullptr, st);
            if (part) launch_rmsnorm_dweight_reduce(part, d, p.rms_blocks, o.drms_weight_out, st);
        }
        if (dw_staged) {
            Span sp(ST_CONVERT, st);
            if (o.dw_dtype == RAPID_DTYPE_BF16) launch_f32_to_bf16(dW32, (bf16_t*)dW_out, d * V, st);
            else launch_f32_add(dW32, (float*)dW_out, d * V, st);
        }
        return check_launch(name);
    }

    // ---- the backward that regenerates the logits (and the fp32 path): forward over the whole batch first.
    // bf16: the generations without gradient (see the cached backward above) come last, and dz, dHidden and dW
    // stop in front of them
    const int32_t* bwd_counts = counts;
    if (dtype == RAPID_DTYPE_BF16 && g_skip_idle.load() && !(clip && clip->o.kl_beta != 0.f)) {
        io.idle.rewards = rewards; io.idle.coef_override = clip ? nullptr : o.coef_override;
        io.idle.idle = at<int32_t>(ws, p.idle); io.idle.len_live = at<int32_t>(ws, p.len_live);
        io.idle.cu_live = at<int32_t>(ws, p.cu_live); io.idle.live_group = at<int32_t>(ws, p.live_group);
        io.group_ids = group_ids;
        bwd_counts = at<int32_t>(ws, p.tab) + CH_LIVE;
    }
    run_forward(p, ws, io, st);

    // generation-level log ratios, clipped-weight group baseline, coefficients and loss
    if (clip) {
        Span sp(ST_ESTIMATOR, st);
        launch_group_advantage(rewards, group_ids, nullptr, nullptr, N, K, 2.f, BASELINE_NORMALIZED, adv, adv64, nullptr, nullptr,
                               nullptr, nullptr, nullptr, dev_status, st, clip->o.adv_eps, clip->o.std_ddof, gruns);
        launch_clip_generations(cl, nullptr, at<double>(ws, p.g64), at<double>(ws, p.tsum), at<double>(ws, p.tmax), dev_status, st);
        launch_clip_finish(at<double>(ws, p.g64), at<double>(ws, p.tsum), at<double>(ws, p.tmax), N, counts, loss_out, clip->diag, st);
        launch_clip_rows(cl, seqc, row_index, counts, 0, p.Mmax_pad, rowg, st);
    } else {
        Span sp(ST_ESTIMATOR, st);
        launch_seq_logratio(logp_cur, logp_behav, mask, N, T, tok_logratio_out, s64, s32, o.eta, o.coef_mode == 1,
                            tsum, tmax, nullptr, dev_status, st);
        launch_group_advantage(rewards, group_ids, nullptr, logp_behav ? s64 : nullptr, N, K, o.eta, o.baseline_mode, adv,
                               adv64, nullptr, nullptr, nullptr, nullptr, nullptr, dev_status, st, 0.f, 0, gruns);
        launch_coefficients(ca, st);
        launch_row_coefficients(g, ca.g64, seqc, row_index, counts, logp_cur, logp_behav, per_token, o.eta,
                                o.coef_mode == 1, 0, p.Mmax_pad, rowg, st);
    }

    // backward, in row chunks
    {
        Span sp(ST_ZERO, st);
        launch_zero_masked_rows(dhidden_out, mask, p.Mmax, d, elem, io.idle.idle, T, st);
    }
    const bool dw_staged = o.dw_dtype == RAPID_DTYPE_BF16;
    float* dW32 = dw_staged ? at<float>(ws, p.dw32) : (float*)dW_out;

    if (dtype == RAPID_DTYPE_BF16) {
        bf16_t* Hc = at<bf16_t>(ws, p.Hc);
        bf16_t* Wvd = at<bf16_t>(ws, p.Wvd);
        bf16_t* Wdv = at<bf16_t>(ws, p.Wdv);
        const bool blocked_wdv = g_blocked_wdv.load() != 0;
        {
            Span sp(ST_PACK, st);
            if (o.w_layout == RAPID_W_DV)
                launch_copy_pad_bf16((const bf16_t*)W, p.V, nullptr, Wdv, p.ldv, p.d, p.V, p.dpadR, p.Vpad,
                                     nullptr, 0, st);
            else
                launch_transpose_pad_bf16((const bf16_t*)W, p.d, Wdv, p.ldv, p.V, p.d, p.Vpad, p.dpadR, nullptr,
                                          0, st);
            if (blocked_wdv)
                launch_block_rows_bf16(Wdv, p.ldv, at<bf16_t>(ws, p.WdvB), p.dpadR, p.Vpad, p.dpadR % 256 == 0 ? 256 : 128, st);
        }
        const int64_t step = p.Mc;
        int chunk = 0;
        for (int64_t m0 = 0; m0 < p.Mmax_pad; m0 += step, ++chunk) {
            const int64_t rows = (p.Mmax_pad - m0) < step ? (p.Mmax_pad - m0) : step;   // multiple of 256
            bf16_t* dz = at<bf16_t>(ws, p.chunk0);
            DzArgs za;
            za.Wvd = Wvd; za.Hc = Hc + m0 * p.ldk; za.dpad = p.dpad; za.ldk = p.ldk; za.ldz = p.ldv;
            za.tilesV = (int)(p.Vpad / 256); za.tilesM = (int)(rows / 256);
            za.V = p.V; za.Vpad = p.Vpad; za.inv_temp = inv_temp; za.m0 = m0;
            za.tokc = tokc; za.lse_c = lse_c; za.rowg = rowg; za.counts = bwd_counts; za.dz = dz; za.gi = g_gi_fwd;
            {
                // like the forward, in sub-blocks of rows whose hidden rows stay in the memory-side cache
                const int64_t sub = (int64_t)g_fwd_block_tiles.load() * 256;
                for (int64_t r0 = 0; r0 < rows; r0 += sub) {
                    const int64_t nrows = (rows - r0) < sub ? (rows - r0) : sub;
                    DzArgs zs = za;
                    zs.Hc = za.Hc + r0 * p.ldk; zs.dz = za.dz + r0 * p.ldv; zs.m0 = m0 + r0;
                    zs.tilesM = (int)(nrows / 256);
                    Span sp(ST_DZ, st);
                    launch_dz(zs, st);
                }
            }
            DhArgs ha;
            ha.Wdv = Wdv; ha.WdvB = blocked_wdv ? at<bf16_t>(ws, p.WdvB) : nullptr; ha.dz = dz; ha.Vpad = p.Vpad; ha.ldv = p.ldv; ha.d = p.d; ha.dpadR = p.dpadR;
            ha.tilesM = (int)(rows / 256); ha.m0 = m0; ha.row_index = row_index; ha.counts = bwd_counts;
            ha.rowc = nullptr;
            const int pace_every = g_pace_every.load();
            ha.pace = pace_every > 0 ? at<unsigned>(ws, p.pace) : nullptr; ha.pace_every = pace_every;
            if (ha.pace) launch_fill_f32((float*)ha.pace, 64, 0.f, st);
            ha.dhidden = (bf16_t*)dhidden_out; ha.gi = g_gi_dh;
            ha.part = g_dh_split.load() ? at<float>(ws, p.dh_part) : nullptr; ha.part_bytes = dh_part_bytes();
            {
                Span sp(ST_DH, st);
                launch_dh(ha, st);
            }
            DwArgs wa;
            wa.dz = dz; wa.Hc = Hc + m0 * p.ldk; wa.Mc = step; wa.ldz = p.ldv; wa.ldH = p.ldk;
            wa.d = p.d; wa.dpadR = p.dpadR; wa.V = p.V; wa.Vpad = p.Vpad; wa.m0 = m0; wa.counts = bwd_counts;
            wa.dW = dW32; wa.w_layout = o.w_layout; wa.beta = (chunk > 0 || o.accumulate_dw) ? 1 : 0; wa.gi = g_gi_dw;
            {
                Span sp(ST_DW, st);
                launch_dw(wa, st);
            }
        }
        if (o.rms_weight) {   // dhidden holds dL/dh of the normalised state: on to dL/dweight and dL/dx
            Span sp(ST_ZERO, st);
            float* part = o.drms_weight_out ? at<float>(ws, p.rms_part) : nullptr;
            if (part) launch_fill_f32(part, p.rms_blocks * d, 0.f, st);
            launch_rmsnorm_backward((const bf16_t*)hidden, (bf16_t*)dhidden_out, d, (const bf16_t*)o.rms_weight, row_index,
                                    counts, at<float>(ws, p.inv_rms), 0, p.Mmax_pad, part, st);
            if (part) launch_rmsnorm_dweight_reduce(part, d, p.rms_blocks, o.drms_weight_out, st);
        }
    } else {
        float* z = at<float>(ws, p.chunk0);
        int chunk = 0;
        Span sp(ST_F32, st);
        for (int64_t m0 = 0; m0 < p.Mmax; m0 += p.Mc, ++chunk) {
            const int64_t rows = (p.Mmax - m0) < p.Mc ? (p.Mmax - m0) : p.Mc;
            F32Gemm gz;
            memset(&gz, 0, sizeof(gz));
            gz.A = (const float*)hidden; gz.sa_i = d; gz.sa_k = 1; gz.a_imap = row_index;
            gz.B = (const float*)W;
            if (o.w_layout == RAPID_W_DV) { gz.sb_k = V; gz.sb_j = 1; } else { gz.sb_k = 1; gz.sb_j = d; }
            gz.C = z; gz.sc_i = V; gz.sc_j = 1;
            gz.I = rows; gz.J = V; gz.Kd = d; gz.beta = 0; gz.counts = counts; gz.i0 = m0; gz.alpha = inv_temp;
            launch_f32_gemm(gz, st);
            launch_f32_dz(z, V, rows, m0, tokc, lse_c, rowg, inv_temp, counts, st);
            // dH[row] = dz[row, :] . W^T
            F32Gemm gh;
            memset(&gh, 0, sizeof(gh));
            gh.A = z; gh.sa_i = V; gh.sa_k = 1;
            gh.B = (const float*)W;   // B(k = v, j = k') = W(k', v)
            if (o.w_layout == RAPID_W_DV) { gh.sb_k = 1; gh.sb_j = V; } else { gh.sb_k = d; gh.sb_j = 1; }
            gh.C = (float*)dhidden_out; gh.sc_i = d; gh.sc_j = 1; gh.c_rows = row_index;
            gh.I = rows; gh.J = d; gh.Kd = V; gh.beta = 0; gh.counts = counts; gh.i0 = m0; gh.alpha = 1.f;
            launch_f32_gemm(gh, st);
            // dW(k', v) += sum_rows H[row, k'] dz[row, v]
            F32Gemm gw;
            memset(&gw, 0, sizeof(gw));
            gw.A = (const float*)hidden; gw.sa_i = 1; gw.sa_k = d; gw.a_kmap = row_index;
            gw.B = z; gw.sb_k = V; gw.sb_j = 1;
            gw.C = dW32;
            if (o.w_layout == RAPID_W_DV) { gw.sc_i = V; gw.sc_j = 1; } else { gw.sc_i = 1; gw.sc_j = d; }
            gw.I = d; gw.J = V; gw.Kd = rows; gw.beta = (chunk > 0 || o.accumulate_dw) ? 1 : 0;
            gw.counts = counts; gw.i0 = m0; gw.limit_k = 1; gw.alpha = 1.f;
            launch_f32_gemm(gw, st);
        }
    }
    if (dw_staged) {
        Span sp(ST_CONVERT, st);
        launch_f32_to_bf16(dW32, (bf16_t*)dW_out, d * V, st);
    }
    return check_launch(name);
}

extern "C" {

int rapid_iw_pg_loss_fwd_bwd(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                             const float* logp_behav, const float* rewards, const int32_t* group_ids, int64_t N,
                             int64_t T, int64_t d, int64_t V, int64_t K, int dtype, const rapid_iw_pg_opts* opts,
                             float* loss_out, void* dhidden_out, void* dW_out, float* logp_cur_out,
                             float* tok_logratio_out, float* seq_logratio_out, float* adv_out,
                             rapid_iw_pg_diag* diag_out, int32_t* dev_status, void* workspace,
                             size_t workspace_bytes, void* stream) {
    rapid_iw_pg_opts o;
    if (opts) o = *opts; else rapid_iw_pg_default_opts(&o);
    return fused_call("rapid_iw_pg_loss_fwd_bwd", hidden, W, tokens, mask, logp_behav, rewards, group_ids, N, T, d, V, K,
                      dtype, o, loss_out, dhidden_out, dW_out, logp_cur_out, tok_logratio_out, seq_logratio_out, adv_out,
                      diag_out, dev_status, workspace, workspace_bytes, stream, nullptr);
}

void rapid_clip_pg_default_opts(rapid_clip_pg_opts* o, int variant) {
    if (!o) return;
    memset(o, 0, sizeof(*o));
    o->eps_low = 0.2f;
    o->eps_high = variant == 1 ? 0.28f : 0.2f;
    o->kl_beta = variant == 1 ? 0.f : 0.04f;
    o->norm_mode = variant == 1 ? 1 : 0;
    o->adv_eps = 1e-4f;
    o->std_ddof = 0;
    o->loss_scale = 1.0f;
    o->temperature = 1.0f;
    o->w_layout = RAPID_W_DV;
    o->dw_dtype = RAPID_DTYPE_F32;
}

int rapid_clip_pg_loss_fwd_bwd(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                               const float* logp_old, const float* logp_ref, const float* rewards,
                               const int32_t* group_ids, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K,
                               int dtype, const rapid_clip_pg_opts* opts, float* loss_out, void* dhidden_out,
                               void* dW_out, float* logp_cur_out, float* adv_out, rapid_clip_pg_diag* diag_out,
                               int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream) {
    ClipSpec cs;
    if (opts) cs.o = *opts; else rapid_clip_pg_default_opts(&cs.o, 0);
    cs.logp_ref = logp_ref;
    cs.diag = diag_out;
    const rapid_clip_pg_opts& c = cs.o;
    if (!(c.eps_low >= 0.f) || !(c.eps_low < 1.f) || !(c.eps_high >= 0.f) || !std::isfinite(c.eps_high) ||
        !(c.kl_beta >= 0.f) || !std::isfinite(c.kl_beta) || !(c.adv_eps >= 0.f) || !std::isfinite(c.adv_eps)) {
        set_error("eps_low must be in [0, 1), eps_high, kl_beta and adv_eps finite and >= 0");
        return RAPID_ERR_SHAPE;
    }
    if (c.norm_mode < 0 || c.norm_mode > 1 || c.std_ddof < 0 || c.std_ddof > 1) {
        set_error("unknown norm_mode / std_ddof");
        return RAPID_ERR_DTYPE;
    }
    if (c.kl_beta != 0.f && !logp_ref) {
        set_error("kl_beta != 0 needs logp_ref");
        return RAPID_ERR_NULL;
    }
    rapid_iw_pg_opts o;     // the options the two calls share
    rapid_iw_pg_default_opts(&o);
    o.loss_scale = c.loss_scale; o.temperature = c.temperature; o.w_layout = c.w_layout; o.dw_dtype = c.dw_dtype;
    o.accumulate_dw = c.accumulate_dw; o.logits_cache = c.logits_cache; o.max_tokens = c.max_tokens;
    return fused_call("rapid_clip_pg_loss_fwd_bwd", hidden, W, tokens, mask, logp_old, rewards, group_ids, N, T, d, V, K,
                      dtype, o, loss_out, dhidden_out, dW_out, logp_cur_out, nullptr, nullptr, adv_out, nullptr, dev_status,
                      workspace, workspace_bytes, stream, &cs);
}

}  // extern "C"
