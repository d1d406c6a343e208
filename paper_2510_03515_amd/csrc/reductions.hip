// Small kernels around the contractions: mask compaction, log-sum-exp merge, generation-level log
// ratios, group advantages, loss/coefficients/diagnostics.  All HBM- or latency-bound; every
// reduction uses a fixed tree so results are bitwise reproducible (no atomics on data).
#include <cmath>

#include "rapid_internal.h"

namespace rapid {

namespace {

constexpr int WAVE = 64;

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ inline double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ inline int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// block-wide reductions for up to 1024 threads; `sm` holds >= 16 doubles
__device__ inline double block_sum(double v, double* sm) {
    v = wave_sum(v);
    const int w = threadIdx.x / WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sm[w] = v;
    __syncthreads();
    double r = 0.0;
    for (int i = 0; i < nw; ++i) r += sm[i];
    return r;
}
__device__ inline double block_max(double v, double* sm) {
    v = wave_max(v);
    const int w = threadIdx.x / WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sm[w] = v;
    __syncthreads();
    double r = sm[0];
    for (int i = 1; i < nw; ++i) r = fmax(r, sm[i]);
    return r;
}

// ------------------------------------------------------------------ compaction of the padding mask
// one wave per generation: number of valid tokens
__global__ void seq_len_kernel(const uint8_t* __restrict__ mask, int64_t N, int64_t T,
                               int32_t* __restrict__ seq_len) {
    const int64_t n = blockIdx.x;
    if (n >= N) return;
    int cnt = 0;
    for (int64_t t = threadIdx.x; t < T; t += WAVE) cnt += mask[n * T + t] != 0;
    cnt = wave_sum_i(cnt);
    if (threadIdx.x == 0) seq_len[n] = cnt;
}

// single block: exclusive prefix sum of seq_len, and the counters M / M rounded up to a row tile.
// The counters never exceed row_cap (the rows the caller's buffers hold): tokens past it are left
// out of everything downstream and RAPID_STATUS_TOKEN_BOUND is set.
__global__ void scan_kernel(const int32_t* __restrict__ seq_len, int64_t N, int32_t* __restrict__ cu,
                            int32_t* __restrict__ counts, int64_t row_cap, int32_t* __restrict__ dev_status) {
    constexpr int PER = 8;   // consecutive entries per thread: 8192 per sweep of the block
    __shared__ int sm[1024];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < N; base += 1024 * PER) {
        const int64_t n0 = base + (int64_t)threadIdx.x * PER;
        int v[PER], mine = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            v[u] = n0 + u < N ? seq_len[n0 + u] : 0;
            mine += v[u];
        }
        sm[threadIdx.x] = mine;
        __syncthreads();
        for (int o = 1; o < 1024; o <<= 1) {   // Hillis-Steele inclusive scan of the threads' sums
            int add = threadIdx.x >= o ? sm[threadIdx.x - o] : 0;
            __syncthreads();
            sm[threadIdx.x] += add;
            __syncthreads();
        }
        const int incl = sm[threadIdx.x];
        int run = carry + incl - mine;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            if (n0 + u < N && cu) cu[n0 + u] = run;
            run += v[u];
        }
        __syncthreads();
        if (threadIdx.x == 1023) carry += incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (cu) cu[N] = carry;
        if (counts) {
            int m = carry;
            if ((int64_t)m > row_cap) {
                m = (int)row_cap;
                if (dev_status) atomicOr(dev_status, RAPID_STATUS_TOKEN_BOUND);
            }
            counts[CNT_M] = m;
            counts[CNT_MR] = (m + ROW_TILE - 1) / ROW_TILE * ROW_TILE;
        }
    }
}

// one wave per generation: flat positions of its valid tokens, in order, from compact row first_row[n]
// on (a negative first row: the generation was left out).  The compact rows come in regions of
// `region` rows; a generation never writes past the end of the region its first row lies in.
__global__ void row_index_kernel(const uint8_t* __restrict__ mask, int64_t N, int64_t T,
                                 const int32_t* __restrict__ first_row, int64_t region,
                                 int32_t* __restrict__ row_index) {
    const int64_t n = blockIdx.x;
    if (n >= N) return;
    int64_t base = first_row[n];
    if (base < 0) return;
    const int64_t limit = (base / region + 1) * region;
    const int lane = threadIdx.x;
    for (int64_t t0 = 0; t0 < T; t0 += WAVE) {
        const int64_t t = t0 + lane;
        const bool v = t < T && mask[n * T + t] != 0;
        const unsigned long long b = __ballot(v);
        const int before = __popcll(b & ((1ull << lane) - 1ull));
        if (v && base + before < limit) row_index[base + before] = (int32_t)(n * T + t);
        base += __popcll(b);
    }
}

// Generations whose coefficient dLoss/dlogp is zero whatever the log-probs turn out to be: every reward of the
// group is exactly 0 (then the weighted baseline of Eq. (5) is 0 too, A_n = R_n - b = 0, in every baseline mode;
// likewise the normalised advantage of the clipped surrogate), or the caller's coefficient override is 0.
// Their rows get no gradient: dHidden rows are zero and they add nothing to dW, so the two gradient
// contractions can leave them out.  Step 1: live_group[g] = 1 for a group with a reward that is not 0.
__global__ void live_groups_kernel(const float* __restrict__ rewards, const int32_t* __restrict__ gid, int64_t N,
                                   int64_t K, int32_t* __restrict__ live_group) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    const float R = rewards[n];
    const int32_t g = gid[n];
    // a reward that is not finite counts as 0 in the estimator as well; equal values from several threads
    if (g >= 0 && g < K && isfinite(R) && R != 0.f) live_group[g] = 1;
}
// Step 2: idle[n], and the generation's length if it is not idle (for the prefix sum the chunk plan uses).
// A generation with a group id outside [0, K) is never idle.
__global__ void idle_generations_kernel(const int32_t* __restrict__ gid, const float* __restrict__ coef_override,
                                        const int32_t* __restrict__ live_group, const int32_t* __restrict__ seq_len,
                                        int64_t N, int64_t K, int32_t* __restrict__ idle,
                                        int32_t* __restrict__ len_live) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    bool z;
    if (coef_override) {
        z = coef_override[n] == 0.f;
    } else {
        const int32_t g = gid[n];
        z = g >= 0 && g < K && live_group[g] == 0;
    }
    idle[n] = z ? 1 : 0;
    len_live[n] = z ? 0 : seq_len[n];
}

// Single block: deals the generations to chunks (see launch_compaction_chunked in rapid_internal.h).
// Thread 0 walks the runs of equal group id in order and fills chunk after chunk; then all threads
// give every generation its chunk and first compact row and count each run's group id once.
// With `idle` (see idle_generations_kernel; cu_live = prefix sum of the other generations' lengths) a chunk's
// rows are ordered: the generations that carry gradient first, in batch order, then the idle ones, so that the
// two gradient contractions stop at CH_LIVE.
__global__ __launch_bounds__(1024) void plan_chunks_kernel(const int32_t* __restrict__ cu,
                                                           const int32_t* __restrict__ cu_live,
                                                           const int32_t* __restrict__ idle,
                                                           const int32_t* __restrict__ gid, int64_t N, int64_t K,
                                                           int64_t Rcap, int Cmax, int32_t* __restrict__ gseen,
                                                           int32_t* __restrict__ tab, int32_t* __restrict__ gen_row0,
                                                           int32_t* __restrict__ gen_chunk,
                                                           int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ dev_status) {
    __shared__ int s_status;
    if (threadIdx.x == 0) {
        int status = 0, c = 0;
        int64_t placed = 0;
        auto close = [&](int64_t g0, int64_t g1, int64_t rows) {
            if (rows > Rcap) rows = Rcap;
            int32_t* e = tab + (int64_t)c * CH_WORDS;
            e[CH_G0] = (int32_t)g0; e[CH_G1] = (int32_t)g1; e[CH_ROWS] = (int32_t)rows;
            e[CH_M] = (int32_t)((int64_t)c * Rcap + rows);
            e[CH_MR] = (int32_t)((int64_t)c * Rcap + (rows + ROW_TILE - 1) / ROW_TILE * ROW_TILE);
            int64_t live = cu_live ? (int64_t)cu_live[g1] - (int64_t)cu_live[g0] : rows;
            if (live > rows) live = rows;           // only when the chunk was cut short (its outputs are unusable then)
            e[CH_LIVE] = (int32_t)((int64_t)c * Rcap + live);
            e[CH_LIVER] = (int32_t)((int64_t)c * Rcap + (live + ROW_TILE - 1) / ROW_TILE * ROW_TILE);
            e[7] = 0;
            placed += rows;
            ++c;
        };
        if (Cmax == 1) {
            const int64_t total = cu[N];
            if (total > Rcap) status |= RAPID_STATUS_TOKEN_BOUND;
            close(0, N, total);
        } else {
            int64_t chunk_g0 = 0, chunk_rows = 0, run0 = 0;
            int run_gid = gid[0];
            bool full = false;
            for (int64_t n = 1; n <= N && !full; ++n) {
                if (n < N && gid[n] == run_gid) continue;
                const int64_t rows = (int64_t)cu[n] - (int64_t)cu[run0];   // the run [run0, n)
                if (rows > Rcap) status |= RAPID_STATUS_GROUP_LAYOUT;      // placed alone, cut at Rcap
                if (run0 > chunk_g0 && chunk_rows + rows > Rcap) {
                    if (c == Cmax - 1) {            // no chunk left: the rest of the batch is left out
                        status |= RAPID_STATUS_TOKEN_BOUND;
                        full = true;
                        break;
                    }
                    close(chunk_g0, run0, chunk_rows);
                    chunk_g0 = run0;
                    chunk_rows = 0;
                }
                chunk_rows += rows;
                run0 = n;
                if (n < N) run_gid = gid[n];
            }
            close(chunk_g0, run0, chunk_rows);      // run0 == N unless the chunks ran out
        }
        while (c < Cmax) close(N, N, 0);            // chunks that stay empty (close() counts c up)
        counts[CNT_M] = (int32_t)placed;
        counts[CNT_MR] = (int32_t)((placed + ROW_TILE - 1) / ROW_TILE * ROW_TILE);
        s_status = status;
    }
    __syncthreads();
    int status = 0;
    for (int64_t n = threadIdx.x; n < N; n += blockDim.x) {
        int c = -1;
        for (int k = 0; k < Cmax; ++k)
            if (n >= tab[k * CH_WORDS + CH_G0] && n < tab[k * CH_WORDS + CH_G1]) { c = k; break; }
        gen_chunk[n] = c;
        int64_t row0 = -1;
        if (c >= 0) {
            const int64_t g0 = tab[c * CH_WORDS + CH_G0], g1 = tab[c * CH_WORDS + CH_G1];
            const int64_t before = (int64_t)cu[n] - (int64_t)cu[g0];            // tokens of the chunk's earlier generations
            if (cu_live) {
                const int64_t live_before = (int64_t)cu_live[n] - (int64_t)cu_live[g0];
                const int64_t live_all = (int64_t)cu_live[g1] - (int64_t)cu_live[g0];
                row0 = (int64_t)c * Rcap + (idle[n] ? live_all + (before - live_before) : live_before);
            } else {
                row0 = (int64_t)c * Rcap + before;
            }
        }
        gen_row0[n] = (int32_t)row0;
        if (Cmax > 1 && (n == 0 || gid[n] != gid[n - 1])) {       // first generation of a run
            const int32_t g = gid[n];
            if (g >= 0 && g < K && atomicAdd(&gseen[g], 1) > 0) status |= RAPID_STATUS_GROUP_LAYOUT;
        }
    }
    if (threadIdx.x == 0) status |= s_status;
    if (status && dev_status) atomicOr(dev_status, status);
}

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
__global__ void fill_f64_kernel(double* p, int64_t n, double v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
__global__ void f32_add_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] += src[i];
}

__global__ void fill_f32_kernel(float* p, int64_t n, float v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// compact token ids and generation ids; out-of-range ids are flagged and replaced by 0
__global__ void gather_tokens_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ row_index,
                                     const int32_t* __restrict__ counts, int64_t row0, int64_t rows_max, int64_t T,
                                     int64_t V, int32_t* __restrict__ tokc, int32_t* __restrict__ seqc,
                                     int32_t* __restrict__ dev_status) {
    const int64_t jl = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t j = row0 + jl;
    const int M = counts[CNT_M], Mr = counts[CNT_MR];
    if (j >= Mr || jl >= rows_max) return;
    int tok = 0, seq = 0;
    if (j < M) {
        const int32_t pos = row_index[j];
        tok = tokens[pos];
        seq = (int32_t)(pos / T);
        if (tok < 0 || tok >= V) {
            tok = 0;
            if (dev_status) atomicOr(dev_status, RAPID_STATUS_BAD_TOKEN);
        }
    }
    tokc[j] = tok;
    seqc[j] = seq;
}

// lse[j] = log sum_p part_sum[p][j] exp(part_max[p][j]) ; logp = zy - lse, scattered to [N,T].
// Four lanes share a column: lane group q (lanes 16 q .. 16 q + 15 of a wave) folds the slots
// [q P/4, (q+1) P/4) of 16 neighbouring columns, then the four (max, sum) pairs of a column are merged in
// the order ((0, 1), (2, 3)).  A thread's loads are a dependent chain of P / 32 batches; one thread per column
// left a 90 000-row chunk with too few threads to cover the memory latency.
__global__ __launch_bounds__(256) void merge_lse_kernel(const float* __restrict__ part_max, const float* __restrict__ part_sum, int P,
                                 int64_t ld_part, const float* __restrict__ zy,
                                 const int32_t* __restrict__ row_index, const int32_t* __restrict__ counts,
                                 int64_t row0, float* __restrict__ lse_c, float* __restrict__ logp_out,
                                 float* __restrict__ lse_out) {
    const int lane = threadIdx.x & 63, q = lane >> 4;
    // 64 columns per block of 256 threads: wave w covers columns 16 w .. 16 w + 15 of the block
    const int64_t jl = (int64_t)blockIdx.x * 64 + (threadIdx.x >> 6) * 16 + (lane & 15);
    const int64_t j = row0 + jl;
    const int M = counts[CNT_M];
    const bool live = j < M;
    // one pass with a running maximum; slots are merged in a fixed order, so the result is reproducible.
    // The weights exp(pm - mx) are fp32 (relative error 1e-7, far below the fp32 rounding of the
    // partial sums themselves), the accumulation fp64.
    float mx = -INFINITY;
    double acc = 0.0;
    constexpr int UN = 8;   // slots loaded ahead of the fold: the loads of a batch are in flight together
    const int p_begin = (int)((int64_t)P * q / 4), p_end = (int)((int64_t)P * (q + 1) / 4);
    if (live) {
        for (int p0 = p_begin; p0 < p_end; p0 += UN) {
            float pmv[UN], psv[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const bool in = p0 + u < p_end;
                pmv[u] = in ? part_max[(int64_t)(p0 + u) * ld_part + jl] : 0.f;
                psv[u] = in ? part_sum[(int64_t)(p0 + u) * ld_part + jl] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const float pm = pmv[u], ps = psv[u];
                if (!(ps > 0.f)) continue;
                if (pm > mx) {
                    acc = acc * (double)__expf(mx - pm) + (double)ps;   // exp(-inf) = 0 on the first slot
                    mx = pm;
                } else {
                    acc += (double)ps * (double)__expf(pm - mx);
                }
            }
        }
    }
    // merge the four lane groups of the column: (0, 1) and (2, 3), then the two results
#pragma unroll
    for (int step = 16; step <= 32; step <<= 1) {
        const float omx = __shfl_xor(mx, step, 64);
        const double oacc = __shfl_xor(acc, step, 64);
        // both partners compute the same merged pair: the lower lane's operand first
        const bool low = (lane & step) == 0;
        const float m0 = low ? mx : omx, m1 = low ? omx : mx;
        const double a0 = low ? acc : oacc, a1 = low ? oacc : acc;
        const float mm = fmaxf(m0, m1);
        double r = 0.0;
        if (a0 > 0.0) r += a0 * (double)__expf(m0 - mm);
        if (a1 > 0.0) r += a1 * (double)__expf(m1 - mm);
        mx = mm;
        acc = r;
    }
    if (!live || q != 0) return;
    const double lse = (double)mx + log(acc);
    const float lse_f = (float)lse;
    lse_c[j] = lse_f;
    const int32_t pos = row_index[j];
    logp_out[pos] = (float)((double)zy[j] - lse);
    if (lse_out) lse_out[pos] = lse_f;
}

// one wave per generation: token-level log ratios and their sum over the generation; for the
// token-level outer weight also sum_t c_{n,t} and max_t log c_{n,t} of the generation's valid tokens
// (c = the token's ratio, clipped at eta if clip_tokens), tsum/tmax may be NULL
__global__ void seq_logratio_kernel(const float* __restrict__ logp_cur, const float* __restrict__ logp_behav,
                                    const uint8_t* __restrict__ mask, int64_t N, int64_t T,
                                    float* __restrict__ tok_lr, double* __restrict__ s64,
                                    float* __restrict__ s32, double log_eta, int clip_tokens,
                                    double* __restrict__ tsum, double* __restrict__ tmax,
                                    const int32_t* __restrict__ gen_range, int32_t* __restrict__ dev_status) {
    const int64_t n = blockIdx.x;
    if (n >= N) return;
    if (gen_range && (n < gen_range[0] || n >= gen_range[1])) return;
    double acc = 0.0, csum = 0.0, cmax = -INFINITY;
    bool bad = false;
    for (int64_t t = threadIdx.x; t < T; t += WAVE) {
        const int64_t i = n * T + t;
        double dlt = 0.0;
        const bool valid = mask[i] != 0;
        if (valid && logp_behav != nullptr) {   // no behaviour log-probs: on-policy, every ratio is 1
            const float lb = logp_behav[i];
            if (isfinite(lb)) dlt = (double)logp_cur[i] - (double)lb;
            else bad = true;
        }
        if (tok_lr) tok_lr[i] = (float)dlt;
        acc += dlt;
        if (valid) {
            const double lc = clip_tokens ? fmin(dlt, log_eta) : dlt;
            csum += exp(lc);
            cmax = fmax(cmax, lc);
        }
    }
    acc = wave_sum(acc);
    if (__any(bad) && threadIdx.x == 0 && dev_status) atomicOr(dev_status, RAPID_STATUS_NONFINITE_LOGP);
    if (tsum) {
        csum = wave_sum(csum);
        cmax = wave_max(cmax);
    }
    if (threadIdx.x == 0) {
        if (s64) s64[n] = acc;
        if (s32) s32[n] = (float)acc;
        if (tsum) {
            tsum[n] = csum;
            tmax[n] = cmax;
        }
    }
}

__device__ inline double clipped_weight(const float* s32, const double* s64, int64_t n, double log_eta) {
    if (s64) return exp(fmin(s64[n], log_eta));
    if (!s32) return 1.0;
    return exp(fmin((double)s32[n], log_eta));
}

// pass 1 over generations: defaults for entries no group owns, and data checks
__global__ void group_init_kernel(const float* __restrict__ rewards, const int32_t* __restrict__ group_ids,
                                  const float* __restrict__ s32, const double* __restrict__ s64, int64_t N,
                                  int64_t K, double log_eta, float* __restrict__ adv, double* __restrict__ adv64,
                                  float* __restrict__ weight, const int32_t* __restrict__ gen_range,
                                  int32_t* __restrict__ dev_status) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    if (gen_range && (n < gen_range[0] || n >= gen_range[1])) return;
    int bits = 0;
    const int32_t k = group_ids[n];
    if (k < 0 || k >= K) bits |= RAPID_STATUS_BAD_GROUP;
    if (!isfinite(rewards[n])) bits |= RAPID_STATUS_NONFINITE_REWARD;
    if (s64 ? isnan(s64[n]) : (s32 && isnan(s32[n]))) bits |= RAPID_STATUS_NONFINITE_LOGP;
    if (bits && dev_status) atomicOr(dev_status, bits);
    adv[n] = 0.f;
    if (adv64) adv64[n] = 0.0;
    if (weight) weight[n] = (float)clipped_weight(s32, s64, n, log_eta);
}

// Where each group lies in the batch: runs[k] = number of maximal runs of group id k, runs[K + k] / runs[2K + k] =
// begin / end of (the last of) them, runs[3K] = 1 if some group has more than one run.  With one run per group,
// which is how a sampler that draws G generations per prompt lays a batch out, the per-group pass below visits
// each generation once instead of once per group.  runs [3K + 1] must be zero on entry.
__global__ void group_runs_kernel(const int32_t* __restrict__ gid, int64_t N, int64_t K, int32_t* __restrict__ runs) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    const int32_t g = gid[n];
    if (g < 0 || g >= K) return;
    if (n == 0 || gid[n - 1] != g) {
        if (atomicAdd(&runs[g], 1) > 0) runs[3 * K] = 1;
        runs[K + g] = (int32_t)n;
    }
    if (n == N - 1 || gid[n + 1] != g) runs[2 * K + g] = (int32_t)(n + 1);
}

// one block per group: size, mean/std of R, clipped-weight baseline, advantages of its members.
// With gen_range only the generations in the range are looked at (the caller guarantees that a group
// lies inside or outside the range as a whole); a group without a member there writes nothing.
__global__ void group_advantage_kernel(const float* __restrict__ rewards, const int32_t* __restrict__ group_ids,
                                       const float* __restrict__ s32, const double* __restrict__ s64, int64_t N,
                                       double log_eta, int baseline_mode, float* __restrict__ adv,
                                       double* __restrict__ adv64, float* __restrict__ gmean,
                                       float* __restrict__ gstd, int32_t* __restrict__ gsize,
                                       const int32_t* __restrict__ gen_range, double adv_eps, int std_ddof,
                                       const int32_t* __restrict__ runs, int64_t K) {
    __shared__ double sm[16];
    const int k = blockIdx.x;
    int64_t n_begin = gen_range ? gen_range[0] : 0, n_end = gen_range ? gen_range[1] : N;
    if (runs && runs[3 * K] == 0) {   // every group is one run of the batch: look at that run only
        const int64_t r0 = runs[k] ? runs[K + k] : 0, r1 = runs[k] ? runs[2 * K + k] : 0;
        n_begin = n_begin > r0 ? n_begin : r0;
        n_end = n_end < r1 ? n_end : r1;
    }
    double cnt = 0.0, sum_r = 0.0, sum_wr = 0.0;
    for (int64_t n = n_begin + threadIdx.x; n < n_end; n += blockDim.x) {
        if (group_ids[n] == k) {
            float r = rewards[n];
            if (!isfinite(r)) r = 0.f;
            cnt += 1.0;
            sum_r += (double)r;
            sum_wr += clipped_weight(s32, s64, n, log_eta) * (double)r;
        }
    }
    cnt = block_sum(cnt, sm);
    sum_r = block_sum(sum_r, sm);
    sum_wr = block_sum(sum_wr, sm);
    if (gen_range && cnt == 0.0) return;   // uniform over the block
    const double mean = cnt > 0.0 ? sum_r / cnt : 0.0;
    double sq = 0.0;
    for (int64_t n = n_begin + threadIdx.x; n < n_end; n += blockDim.x) {
        if (group_ids[n] == k) {
            float r = rewards[n];
            if (!isfinite(r)) r = 0.f;
            const double dlt = (double)r - mean;
            sq += dlt * dlt;
            double b;
            if (baseline_mode == BASELINE_NORMALIZED) {
                continue;                      // needs the group's std: third pass below
            } else if (baseline_mode == 0) {
                b = sum_wr / cnt;
            } else {
                const double rest = sum_wr - clipped_weight(s32, s64, n, log_eta) * (double)r;
                if (baseline_mode == 1) b = rest / cnt;
                else b = cnt > 1.0 ? rest / (cnt - 1.0) : 0.0;
            }
            adv[n] = (float)((double)r - b);
            if (adv64) adv64[n] = (double)r - b;
        }
    }
    sq = block_sum(sq, sm);
    if (baseline_mode == BASELINE_NORMALIZED) {   // (R - mean) / (std + eps); equal rewards give 0
        const double den = cnt - (double)std_ddof;
        const double sd = den > 0.0 ? sqrt(sq / den) : 0.0;
        for (int64_t n = n_begin + threadIdx.x; n < n_end; n += blockDim.x) {
            if (group_ids[n] == k) {
                float r = rewards[n];
                if (!isfinite(r)) r = 0.f;
                const double num = (double)r - mean;
                const double a = num != 0.0 ? num / (sd + adv_eps) : 0.0;
                adv[n] = (float)a;
                if (adv64) adv64[n] = a;
            }
        }
    }
    if (threadIdx.x == 0) {
        if (gsize) gsize[k] = (int32_t)cnt;
        if (gmean) gmean[k] = (float)mean;
        if (gstd) gstd[k] = (float)(cnt > 0.0 ? sqrt(sq / cnt) : 0.0);
    }
}

// single block: coefficients g_n, the loss, diagnostics (the three uses are described at CoefArgs).
// Generation-level outer weight (tsum NULL): g_n = -(loss_scale/N) c_n A_n, loss = sum_n g_n.
// Token-level (tsum, tmax given): g_n is the generation's factor -(loss_scale/N) A_n, a token's
// coefficient is g_n c_{n,t}, and loss = sum_n g_n sum_t c_{n,t}.  g64 keeps g_n in double for the
// per-row pass.
__global__ void coefficients_kernel(CoefArgs a, double log_eta, double log_loss_scale) {
    __shared__ double sm[16];
    const int64_t N = a.N;
    const double logN = log((double)N);
    const bool per_token = a.tsum != nullptr && !a.coef_override;
    const bool chunk_pass = a.gen_range != nullptr;
    const int64_t n_begin = chunk_pass ? a.gen_range[0] : 0, n_end = chunk_pass ? a.gen_range[1] : N;
    auto advantage = [&](int64_t n) { return a.adv64 ? a.adv64[n] : (double)a.adv[n]; };
    double lam = 0.0;
    if (!a.coef_override && a.normalized) {
        double mx = -INFINITY;
        for (int64_t n = n_begin + threadIdx.x; n < n_end; n += blockDim.x) {
            const double av = advantage(n);
            if (av != 0.0) {
                const double lc = per_token ? a.tmax[n] : (a.coef_mode == 0 ? a.s64[n] : fmin(a.s64[n], log_eta));
                mx = fmax(mx, lc + log(fabs(av)) + log_loss_scale - logN);   // -inf for a generation without tokens
            }
        }
        mx = block_max(mx, sm);
        if (chunk_pass) {
            const double before = a.lam_state[0];        // -inf: no chunk has carried a coefficient yet
            const double now = fmax(before, mx);
            __syncthreads();                             // everybody has read the old state
            if (threadIdx.x == 0) {
                a.lam_state[0] = now;
                a.lam_chunk[0] = now;
                a.beta_out[0] = (before == -INFINITY) ? 1.f : (float)exp(before - now);
            }
            mx = now;
        }
        lam = (mx == -INFINITY) ? 0.0 : mx;
    } else if (chunk_pass && threadIdx.x == 0) {
        a.lam_state[0] = 0.0;
        a.lam_chunk[0] = 0.0;
        a.beta_out[0] = 1.f;
    }
    double loss = 0.0, slw = 0.0, salw = 0.0, maxs = 0.0, nclip = 0.0;
    for (int64_t n = n_begin + threadIdx.x; n < n_end; n += blockDim.x) {
        const double s = a.s64[n];
        double gn;
        if (a.coef_override) {
            gn = (double)a.coef_override[n];
        } else {
            const double av = advantage(n);
            if (av != 0.0) {
                const double lc = per_token ? 0.0 : (a.coef_mode == 0 ? s : fmin(s, log_eta));
                gn = (av > 0.0 ? -1.0 : 1.0) * exp(lc + log(fabs(av)) + log_loss_scale - logN - lam);
            } else {
                gn = 0.0;
            }
        }
        if (a.write_g) {
            a.g[n] = (float)gn;
            a.g64[n] = gn;
        }
        loss += per_token ? (gn != 0.0 ? gn * a.tsum[n] : 0.0) : gn;
        const double lw = fmin(s, log_eta);
        slw += lw;
        salw += fabs(lw);
        maxs = fmax(maxs, fabs(s));
        nclip += s > log_eta ? 1.0 : 0.0;
    }
    if (chunk_pass) return;
    loss = block_sum(loss, sm);
    slw = block_sum(slw, sm);
    salw = block_sum(salw, sm);
    nclip = block_sum(nclip, sm);
    maxs = block_max(maxs, sm);
    if (threadIdx.x == 0) {
        a.loss_out[0] = (float)loss;
        if (a.diag) {
            a.diag->n_tokens = a.counts[CNT_M];
            a.diag->n_clipped = (int32_t)nclip;
            a.diag->n_sequences = (int32_t)N;
            a.diag->mean_log_w = (float)(slw / (double)N);
            a.diag->mean_abs_log_w = (float)(salw / (double)N);
            a.diag->max_abs_s = (float)maxs;
            a.diag->grad_log_scale = (float)lam;
        }
    }
}

// the coefficient dL/dlogp of every compact token row: the generation's g_n, times the token's own
// (clipped) ratio for the token-level outer weight; 0 for the padding rows up to the row-tile boundary
__global__ void row_coefficients_kernel(const float* __restrict__ g, const double* __restrict__ g64,
                                        const int32_t* __restrict__ seqc, const int32_t* __restrict__ row_index,
                                        const int32_t* __restrict__ counts, const float* __restrict__ logp_cur,
                                        const float* __restrict__ logp_behav, int per_token, double log_eta,
                                        int clip_tokens, int64_t row0, float* __restrict__ rowg) {
    const int64_t j = row0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int M = counts[CNT_M], Mr = counts[CNT_MR];
    if (j >= Mr) return;
    float v = 0.f;
    if (j < M) {
        const int32_t n = seqc[j];
        if (!per_token) {
            v = g[n];
        } else {
            double dlt = 0.0;
            if (logp_behav != nullptr) {
                const int32_t pos = row_index[j];
                const float lb = logp_behav[pos];
                if (isfinite(lb)) dlt = (double)logp_cur[pos] - (double)lb;
            }
            v = (float)(g64[n] * exp(clip_tokens ? fmin(dlt, log_eta) : dlt));
        }
    }
    rowg[j] = v;
}

// zero the gradient rows of masked positions, and of every position of an idle generation (idle may be
// NULL): one block per position
__global__ void zero_masked_rows_kernel(uint32_t* __restrict__ dh, const uint8_t* __restrict__ mask,
                                        int64_t rows, int64_t words_per_row, const int32_t* __restrict__ idle,
                                        int64_t T) {
    const int64_t r = blockIdx.x;
    if (r >= rows || (mask[r] != 0 && !(idle && idle[r / T]))) return;
    uint32_t* p = dh + r * words_per_row;
    for (int64_t i = threadIdx.x; i < words_per_row; i += blockDim.x) p[i] = 0u;
}

// one block per position of [N, T]: a valid position's bf16 gradient row times
// exp(lam_chunk[chunk of its generation] - lam_final); rows whose factor is 1 are left alone
__global__ void rescale_rows_kernel(bf16_t* __restrict__ dh, const uint8_t* __restrict__ mask, int64_t T, int64_t d,
                                    const int32_t* __restrict__ gen_chunk, const double* __restrict__ lam_chunk,
                                    const double* __restrict__ lam_state) {
    const int64_t r = blockIdx.x;
    if (mask[r] == 0) return;
    const int c = gen_chunk[r / T];
    if (c < 0) return;
    const double dl = lam_chunk[c] - lam_state[0];
    if (dl == 0.0 || !(dl < 0.0)) return;         // also skips a state that never left -inf (no coefficient anywhere)
    const float f = (float)exp(dl);
    bf16_t* p = dh + r * d;
    for (int64_t i = threadIdx.x; i < d; i += blockDim.x) {
        const float v = __builtin_bit_cast(float, (uint32_t)p[i] << 16) * f;
        const __bf16 o = (__bf16)v;
        p[i] = __builtin_bit_cast(bf16_t, o);
    }
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const __bf16 b = (__bf16)src[i];
    dst[i] = __builtin_bit_cast(unsigned short, b);
}

inline unsigned blocks_for(int64_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

}  // namespace

void launch_compaction(const uint8_t* mask, int64_t N, int64_t T, int32_t* seq_len, int32_t* cu_seqlen,
                       int32_t* row_index, int32_t* counts, int64_t row_cap, int32_t* dev_status, hipStream_t st) {
    seq_len_kernel<<<(unsigned)N, WAVE, 0, st>>>(mask, N, T, seq_len);
    scan_kernel<<<1, 1024, 0, st>>>(seq_len, N, cu_seqlen, counts, row_cap, dev_status);
    if (row_index) row_index_kernel<<<(unsigned)N, WAVE, 0, st>>>(mask, N, T, cu_seqlen, INT64_MAX / 4, row_index);
}

void launch_compaction_chunked(const uint8_t* mask, const int32_t* group_ids, int64_t N, int64_t T, int64_t K,
                               int64_t Rcap, int Cmax, int32_t* seq_len, int32_t* cu_seqlen, int32_t* tab,
                               int32_t* gen_row0, int32_t* gen_chunk, int32_t* gseen, int32_t* row_index,
                               int32_t* counts, int32_t* dev_status, const IdleArgs& z, hipStream_t st) {
    seq_len_kernel<<<(unsigned)N, WAVE, 0, st>>>(mask, N, T, seq_len);
    scan_kernel<<<1, 1024, 0, st>>>(seq_len, N, cu_seqlen, nullptr, INT64_MAX, nullptr);
    if (z.idle) {
        if (!z.coef_override) {
            launch_fill_i32(z.live_group, K, 0, st);
            live_groups_kernel<<<blocks_for(N, 256), 256, 0, st>>>(z.rewards, group_ids, N, K, z.live_group);
        }
        idle_generations_kernel<<<blocks_for(N, 256), 256, 0, st>>>(group_ids, z.coef_override, z.live_group, seq_len, N, K,
                                                                    z.idle, z.len_live);
        scan_kernel<<<1, 1024, 0, st>>>(z.len_live, N, z.cu_live, nullptr, INT64_MAX, nullptr);
    }
    if (Cmax > 1) launch_fill_i32(gseen, K, 0, st);
    plan_chunks_kernel<<<1, 1024, 0, st>>>(cu_seqlen, z.idle ? z.cu_live : nullptr, z.idle, group_ids, N, K, Rcap, Cmax, gseen,
                                           tab, gen_row0, gen_chunk, counts, dev_status);
    row_index_kernel<<<(unsigned)N, WAVE, 0, st>>>(mask, N, T, gen_row0, Rcap, row_index);
}

void launch_fill_f32(float* p, int64_t n, float v, hipStream_t st) {
    if (n > 0) fill_f32_kernel<<<blocks_for(n, 256), 256, 0, st>>>(p, n, v);
}
void launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st) {
    if (n > 0) fill_i32_kernel<<<blocks_for(n, 256), 256, 0, st>>>(p, n, v);
}
void launch_fill_f64(double* p, int64_t n, double v, hipStream_t st) {
    if (n > 0) fill_f64_kernel<<<blocks_for(n, 256), 256, 0, st>>>(p, n, v);
}
void launch_f32_add(const float* src, float* dst, int64_t n, hipStream_t st) {
    if (n > 0) f32_add_kernel<<<blocks_for(n, 256), 256, 0, st>>>(src, dst, n);
}

void launch_gather_tokens(const int32_t* tokens, const int32_t* row_index, const int32_t* counts, int64_t row0,
                          int64_t rows_max, int64_t T, int64_t V, int32_t* tokc, int32_t* seqc,
                          int32_t* dev_status, hipStream_t st) {
    if (rows_max > 0)
        gather_tokens_kernel<<<blocks_for(rows_max, 256), 256, 0, st>>>(tokens, row_index, counts, row0, rows_max, T, V,
                                                                        tokc, seqc, dev_status);
}

void launch_merge_lse(const float* part_max, const float* part_sum, int P, int64_t ld_part, const float* zy,
                      const int32_t* row_index, const int32_t* counts, int64_t row0, int64_t rows_max, float* lse_c,
                      float* logp_out, float* lse_out, hipStream_t st) {
    if (rows_max > 0)
        merge_lse_kernel<<<blocks_for(rows_max, 64), 256, 0, st>>>(part_max, part_sum, P, ld_part, zy, row_index,
                                                                    counts, row0, lse_c, logp_out, lse_out);
}

void launch_seq_logratio(const float* logp_cur, const float* logp_behav, const uint8_t* mask, int64_t N,
                         int64_t T, float* tok_logratio_out, double* s64, float* s32, float eta, int clip_tokens,
                         double* tsum, double* tmax, const int32_t* gen_range, int32_t* dev_status, hipStream_t st) {
    const double log_eta = (eta > 0.f && std::isfinite(eta)) ? log((double)eta) : (double)INFINITY;
    seq_logratio_kernel<<<(unsigned)N, WAVE, 0, st>>>(logp_cur, logp_behav, mask, N, T, tok_logratio_out, s64,
                                                      s32, log_eta, clip_tokens, tsum, tmax, gen_range, dev_status);
}

void launch_group_advantage(const float* rewards, const int32_t* group_ids, const float* s32, const double* s64,
                            int64_t N, int64_t K, float eta, int baseline_mode, float* adv, double* adv64,
                            float* weight, float* gmean, float* gstd, int32_t* gsize, const int32_t* gen_range,
                            int32_t* dev_status, hipStream_t st, float adv_eps, int std_ddof, const int32_t* runs) {
    const double log_eta = (eta > 0.f && std::isfinite(eta)) ? log((double)eta) : (double)INFINITY;
    group_init_kernel<<<blocks_for(N, 256), 256, 0, st>>>(rewards, group_ids, s32, s64, N, K, log_eta, adv, adv64,
                                                          weight, gen_range, dev_status);
    group_advantage_kernel<<<(unsigned)K, 256, 0, st>>>(rewards, group_ids, s32, s64, N, log_eta, baseline_mode, adv,
                                                        adv64, gmean, gstd, gsize, gen_range, (double)adv_eps, std_ddof,
                                                        runs, K);
}

void launch_group_runs(const int32_t* group_ids, int64_t N, int64_t K, int32_t* runs, hipStream_t st) {
    launch_fill_i32(runs, 3 * K + 1, 0, st);
    group_runs_kernel<<<blocks_for(N, 256), 256, 0, st>>>(group_ids, N, K, runs);
}

// ---- the token-level clipped surrogate of the GRPO / DAPO loss steps ---------------------------
namespace {

struct ClipToken { double loss, dlogp, kl; bool clipped; };

// one valid token: omega (surr - beta kl) and its derivative with respect to the current log-prob
__device__ inline ClipToken clip_token(const ClipArgs& a, int64_t i, double adv, double omega, bool* bad) {
    const double cur = (double)a.logp_cur[i];
    double dlt = 0.0;
    if (a.logp_old) {
        const float lo = a.logp_old[i];
        if (isfinite(lo)) dlt = cur - (double)lo; else *bad = true;
    }
    const double r = exp(dlt);
    const double rc = fmin(fmax(r, 1.0 - (double)a.eps_low), 1.0 + (double)a.eps_high);
    const double unclipped = r * adv, clipped = rc * adv;
    ClipToken t;
    t.clipped = unclipped > clipped;
    const double surr = t.clipped ? clipped : unclipped;
    const double dsurr = t.clipped ? 0.0 : unclipped;
    double kl = 0.0, dkl = 0.0;
    if (a.kl_beta != 0.f && a.logp_ref) {
        const float lr = a.logp_ref[i];
        if (isfinite(lr)) {
            const double dref = (double)lr - cur;
            const double e = exp(dref);
            kl = e - dref - 1.0;
            dkl = 1.0 - e;
        } else {
            *bad = true;
        }
    }
    t.kl = kl;
    t.loss = -omega * (surr - (double)a.kl_beta * kl);
    t.dlogp = -omega * (dsurr - (double)a.kl_beta * dkl);
    return t;
}

__device__ inline double clip_omega(const ClipArgs& a, int64_t n) {
    if (a.norm_mode == 0) {
        const int L = a.seq_len[n];
        return L > 0 ? (double)a.loss_scale / ((double)a.N * (double)L) : 0.0;
    }
    const int M = a.counts[CNT_M];
    return M > 0 ? (double)a.loss_scale / (double)M : 0.0;
}

__global__ void clip_rows_kernel(ClipArgs a, const int32_t* __restrict__ seqc, const int32_t* __restrict__ row_index,
                                 const int32_t* __restrict__ row_counts, int64_t row0, float* __restrict__ rowg) {
    const int64_t j = row0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int M = row_counts[CNT_M], Mr = row_counts[CNT_MR];
    if (j >= Mr) return;
    float v = 0.f;
    if (j < M) {
        const int32_t n = seqc[j];
        bool bad = false;
        v = (float)clip_token(a, row_index[j], a.adv64[n], clip_omega(a, n), &bad).dlogp;
    }
    rowg[j] = v;
}

// one wave per generation
__global__ void clip_generations_kernel(ClipArgs a, const int32_t* __restrict__ gen_range, double* __restrict__ loss_n,
                                        double* __restrict__ clipped_n, double* __restrict__ kl_n,
                                        int32_t* __restrict__ dev_status) {
    const int64_t n = blockIdx.x;
    if (n >= a.N) return;
    if (gen_range && (n < gen_range[0] || n >= gen_range[1])) return;
    const double omega = clip_omega(a, n), adv = a.adv64[n];
    double loss = 0.0, ncl = 0.0, kl = 0.0;
    bool bad = false;
    for (int64_t t = threadIdx.x; t < a.T; t += WAVE) {
        const int64_t i = n * a.T + t;
        if (a.mask[i] == 0) continue;
        const ClipToken tk = clip_token(a, i, adv, omega, &bad);
        loss += tk.loss;
        ncl += tk.clipped ? 1.0 : 0.0;
        kl += tk.kl;
    }
    loss = wave_sum(loss);
    ncl = wave_sum(ncl);
    kl = wave_sum(kl);
    if (__any(bad) && threadIdx.x == 0 && dev_status) atomicOr(dev_status, RAPID_STATUS_NONFINITE_LOGP);
    if (threadIdx.x == 0) {
        loss_n[n] = loss;
        clipped_n[n] = ncl;
        kl_n[n] = kl;
    }
}

__global__ void clip_finish_kernel(const double* __restrict__ loss_n, const double* __restrict__ clipped_n,
                                   const double* __restrict__ kl_n, int64_t N, const int32_t* __restrict__ counts,
                                   float* __restrict__ loss_out, rapid_clip_pg_diag* __restrict__ diag) {
    __shared__ double sm[16];
    double loss = 0.0, ncl = 0.0, kl = 0.0;
    for (int64_t n = threadIdx.x; n < N; n += blockDim.x) {
        loss += loss_n[n];
        ncl += clipped_n[n];
        kl += kl_n[n];
    }
    loss = block_sum(loss, sm);
    ncl = block_sum(ncl, sm);
    kl = block_sum(kl, sm);
    if (threadIdx.x == 0) {
        loss_out[0] = (float)loss;
        if (diag) {
            const int M = counts[CNT_M];
            diag->n_tokens = M;
            diag->n_clipped = (int64_t)ncl;
            diag->n_sequences = (int32_t)N;
            diag->mean_kl = M > 0 ? (float)(kl / (double)M) : 0.f;
        }
    }
}

}  // namespace

void launch_clip_rows(const ClipArgs& a, const int32_t* seqc, const int32_t* row_index, const int32_t* row_counts,
                      int64_t row0, int64_t rows_max, float* rowg, hipStream_t st) {
    if (rows_max > 0)
        clip_rows_kernel<<<blocks_for(rows_max, 256), 256, 0, st>>>(a, seqc, row_index, row_counts, row0, rowg);
}
void launch_clip_generations(const ClipArgs& a, const int32_t* gen_range, double* loss_n, double* clipped_n, double* kl_n,
                             int32_t* dev_status, hipStream_t st) {
    clip_generations_kernel<<<(unsigned)a.N, WAVE, 0, st>>>(a, gen_range, loss_n, clipped_n, kl_n, dev_status);
}
void launch_clip_finish(const double* loss_n, const double* clipped_n, const double* kl_n, int64_t N, const int32_t* counts,
                        float* loss_out, rapid_clip_pg_diag* diag, hipStream_t st) {
    clip_finish_kernel<<<1, 1024, 0, st>>>(loss_n, clipped_n, kl_n, N, counts, loss_out, diag);
}

void launch_coefficients(const CoefArgs& a, hipStream_t st) {
    const double log_eta = (a.eta > 0.f && std::isfinite(a.eta)) ? log((double)a.eta) : (double)INFINITY;
    coefficients_kernel<<<1, 1024, 0, st>>>(a, log_eta, log((double)a.loss_scale));
}

void launch_row_coefficients(const float* g, const double* g64, const int32_t* seqc, const int32_t* row_index,
                             const int32_t* counts, const float* logp_cur, const float* logp_behav, int per_token,
                             float eta, int clip_tokens, int64_t row0, int64_t rows_max, float* rowg, hipStream_t st) {
    const double log_eta = (eta > 0.f && std::isfinite(eta)) ? log((double)eta) : (double)INFINITY;
    if (rows_max > 0)
        row_coefficients_kernel<<<blocks_for(rows_max, 256), 256, 0, st>>>(g, g64, seqc, row_index, counts, logp_cur,
                                                                           logp_behav, per_token, log_eta,
                                                                           clip_tokens, row0, rowg);
}

void launch_rescale_rows(void* dhidden, const uint8_t* mask, int64_t N, int64_t T, int64_t d, const int32_t* gen_chunk,
                         const double* lam_chunk, const double* lam_state, hipStream_t st) {
    rescale_rows_kernel<<<(unsigned)(N * T), 128, 0, st>>>((bf16_t*)dhidden, mask, T, d, gen_chunk, lam_chunk, lam_state);
}

void launch_zero_masked_rows(void* dhidden, const uint8_t* mask, int64_t rows, int64_t d, int elem_bytes,
                             const int32_t* idle, int64_t T, hipStream_t st) {
    // d * elem_bytes is a multiple of 4 for every accepted shape (bf16 needs d % 8 == 0)
    zero_masked_rows_kernel<<<(unsigned)rows, 128, 0, st>>>((uint32_t*)dhidden, mask, rows,
                                                            d * elem_bytes / 4, idle, T);
}

// master -= lr * grad; optionally also the updated weights in the contraction dtype
__global__ void sgd_step_kernel(float* __restrict__ master, const float* __restrict__ grad, int64_t n, float lr,
                                void* __restrict__ w_out, int dtype) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float w = master[i] - lr * grad[i];
    master[i] = w;
    if (w_out) {
        if (dtype == RAPID_DTYPE_BF16) {
            const __bf16 r = (__bf16)w;
            ((bf16_t*)w_out)[i] = __builtin_bit_cast(bf16_t, r);
        } else {
            ((float*)w_out)[i] = w;
        }
    }
}
void launch_sgd_step(float* master, const float* grad, int64_t n, float lr, void* w_out, int dtype, hipStream_t st) {
    if (n > 0) sgd_step_kernel<<<blocks_for(n, 256), 256, 0, st>>>(master, grad, n, lr, w_out, dtype);
}

// AdamW: bias corrections 1 - beta^step are formed on the host in double
__global__ void adamw_step_kernel(float* __restrict__ master, const float* __restrict__ grad, float* __restrict__ m,
                                  float* __restrict__ v, int64_t n, float lr, float beta1, float beta2, float eps,
                                  float weight_decay, float inv_bc1, float inv_bc2, void* __restrict__ w_out, int dtype) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float g = grad[i];
    const float mi = beta1 * m[i] + (1.f - beta1) * g;
    const float vi = beta2 * v[i] + (1.f - beta2) * g * g;
    m[i] = mi;
    v[i] = vi;
    const float w0 = master[i];
    const float w = w0 - lr * ((mi * inv_bc1) / (sqrtf(vi * inv_bc2) + eps) + weight_decay * w0);
    master[i] = w;
    if (w_out) {
        if (dtype == RAPID_DTYPE_BF16) {
            const __bf16 r = (__bf16)w;
            ((bf16_t*)w_out)[i] = __builtin_bit_cast(bf16_t, r);
        } else {
            ((float*)w_out)[i] = w;
        }
    }
}
void launch_adamw_step(float* master, const float* grad, float* m, float* v, int64_t n, float lr, float beta1, float beta2,
                       float eps, float weight_decay, int64_t step, void* w_out, int dtype, hipStream_t st) {
    const float inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    const float inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    if (n > 0)
        adamw_step_kernel<<<blocks_for(n, 256), 256, 0, st>>>(master, grad, m, v, n, lr, beta1, beta2, eps, weight_decay,
                                                              inv_bc1, inv_bc2, w_out, dtype);
}

void launch_f32_to_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t st) {
    if (n > 0) f32_to_bf16_kernel<<<blocks_for(n, 256), 256, 0, st>>>(src, dst, n);
}

}  // namespace rapid
