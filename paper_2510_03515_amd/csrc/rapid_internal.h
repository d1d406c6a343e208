// Internal declarations shared by the translation units of librapid_hip.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rapid.h"

namespace rapid {

typedef unsigned short bf16_t;  // raw bf16 bits in memory

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Leading dimension (bf16 elements) for a row of x elements (x a multiple of 64): one extra
// 128-byte line when the row would otherwise span an even number of lines.  Consecutive rows of an
// operand tile are read for the same k at the same time; with an odd line stride they fall on
// different L2 / HBM channels instead of piling onto one or two.
static inline int64_t padded_ld(int64_t x) { return ((x / 64) % 2 == 0) ? x + 64 : x; }

// device counters written by the compaction step: [0] = M (valid tokens), [1] = M rounded up to 256
enum { CNT_M = 0, CNT_MR = 1, CNT_WORDS = 64 };

// One entry of the chunk table of the cached backward (int32 x CH_WORDS per chunk): words 0 and 1 are
// laid out like the counters above, so a kernel that is given `table + CH_WORDS * c` as its counters
// works on chunk c alone.  Chunk c owns the compact rows [c * Rcap, c * Rcap + rows).
enum { CH_M = 0,      // end of the chunk's valid rows (absolute compact row index)
       CH_MR = 1,     // that end rounded up to a row tile
       CH_G0 = 2,     // first generation of the chunk
       CH_G1 = 3,     // one past its last generation
       CH_ROWS = 4,   // valid rows
       CH_LIVE = 5,   // end of the rows that carry gradient (they come first; see IdleArgs); CH_LIVE, CH_LIVER lie
       CH_LIVER = 6,  // like CNT_M, CNT_MR: a kernel given tab + CH_LIVE as its counters stops at them
       CH_WORDS = 8 };

constexpr int ROW_TILE = 256;  // compact rows are padded to this
constexpr int K_TILE = 64;     // contraction tile of the MFMA kernels (bf16 elements)

// ---- reductions.hip ---------------------------------------------------------------------------
// counts (optional): M and M rounded up to a row tile, both clipped to row_cap (sets RAPID_STATUS_TOKEN_BOUND)
void launch_compaction(const uint8_t* mask, int64_t N, int64_t T, int32_t* seq_len, int32_t* cu_seqlen,
                       int32_t* row_index, int32_t* counts, int64_t row_cap, int32_t* dev_status, hipStream_t st);
// Compaction for the cached backward: sequence lengths and their prefix sum as above, then the
// generations are dealt to at most Cmax chunks of at most Rcap compact rows each, whole groups
// (maximal runs of equal group id) at a time, in order, each chunk as full as it gets; chunk c's
// rows start at compact row c * Rcap.  Writes the chunk table `tab` [Cmax][CH_WORDS], gen_row0 [N]
// (compact row of each generation's first token, -1 for a generation that was left out),
// gen_chunk [N], row_index [Cmax * Rcap] and counts[CNT_M] = the tokens that were placed.
// Cmax == 1: one chunk takes every generation, groups may lie anywhere; tokens past Rcap are left
// out (RAPID_STATUS_TOKEN_BOUND).  Cmax > 1: a group whose members are not adjacent, or whose tokens
// exceed Rcap, sets RAPID_STATUS_GROUP_LAYOUT; more chunks than Cmax sets RAPID_STATUS_TOKEN_BOUND.
// gseen [K] is scratch.
// IdleArgs (idle == NULL: off): generations whose coefficient is zero whatever their log-probs are (all rewards
// of the group exactly 0, or a coefficient override of 0) are marked in idle [N] and placed behind the others
// inside their chunk; the chunk's CH_LIVE / CH_LIVER say where the rows that carry gradient end.
struct IdleArgs {
    const float* rewards = nullptr;        // [N]
    const float* coef_override = nullptr;  // [N] or NULL; if given it alone decides
    int32_t* idle = nullptr;               // out [N]
    int32_t* len_live = nullptr;           // scratch [N]
    int32_t* cu_live = nullptr;            // scratch [N + 1]
    int32_t* live_group = nullptr;         // scratch [K]
};
void launch_compaction_chunked(const uint8_t* mask, const int32_t* group_ids, int64_t N, int64_t T, int64_t K,
                               int64_t Rcap, int Cmax, int32_t* seq_len, int32_t* cu_seqlen, int32_t* tab,
                               int32_t* gen_row0, int32_t* gen_chunk, int32_t* gseen, int32_t* row_index,
                               int32_t* counts, int32_t* dev_status, const IdleArgs& z, hipStream_t st);
void launch_fill_f32(float* p, int64_t n, float v, hipStream_t st);
// compact rows [row0, row0 + rows_max) (those below counts[CNT_MR])
void launch_gather_tokens(const int32_t* tokens, const int32_t* row_index, const int32_t* counts, int64_t row0,
                          int64_t rows_max, int64_t T, int64_t V, int32_t* tokc, int32_t* seqc,
                          int32_t* dev_status, hipStream_t st);
// lse/logp from per-slot partial (max, sumexp) and the gathered logit, compact rows [row0, row0 + rows_max);
// the partials of row j sit at column j - row0
void launch_merge_lse(const float* part_max, const float* part_sum, int P, int64_t ld_part,
                      const float* zy, const int32_t* row_index, const int32_t* counts, int64_t row0,
                      int64_t rows_max, float* lse_c, float* logp_out, float* lse_out, hipStream_t st);
// The estimator kernels take `gen_range` (device, two words: first generation and one past the last; NULL =
// all N): they then touch only those generations.
// tsum/tmax (NULL or [N]): per generation, sum and log-maximum of its tokens' (clipped if clip_tokens) ratios
void launch_seq_logratio(const float* logp_cur, const float* logp_behav, const uint8_t* mask, int64_t N,
                         int64_t T, float* tok_logratio_out, double* s64, float* s32, float eta, int clip_tokens,
                         double* tsum, double* tmax, const int32_t* gen_range, int32_t* dev_status, hipStream_t st);
// weights from s64 if given, else from s32, else 1; adv64 (NULL or [N]): the advantages before rounding to float.
// baseline_mode 0..2 as in rapid.h; BASELINE_NORMALIZED: adv = (R - group mean) / (group std + adv_eps), the std
// with divisor N_k - std_ddof (no weights).
constexpr int BASELINE_NORMALIZED = 3;
void launch_group_advantage(const float* rewards, const int32_t* group_ids, const float* s32, const double* s64,
                            int64_t N, int64_t K, float eta, int baseline_mode, float* adv, double* adv64,
                            float* weight, float* gmean, float* gstd, int32_t* gsize, const int32_t* gen_range,
                            int32_t* dev_status, hipStream_t st, float adv_eps = 0.f, int std_ddof = 0,
                            const int32_t* runs = nullptr);
// runs [3K + 1] (see group_runs_kernel): where each group lies in the batch; given to launch_group_advantage it
// lets a group that is one run of the batch look at that run alone
void launch_group_runs(const int32_t* group_ids, int64_t N, int64_t K, int32_t* runs, hipStream_t st);

// Token-level clipped surrogate with KL penalty (the loss step of the GRPO / DAPO baselines).
struct ClipArgs {
    const float* logp_cur; const float* logp_old; const float* logp_ref;   // [N,T]; old NULL: ratios 1; ref NULL: no KL term
    const uint8_t* mask; const double* adv64; const int32_t* seq_len; const int32_t* counts;   // counts[CNT_M]: tokens of the call
    int64_t N, T;
    float eps_low, eps_high, kl_beta, loss_scale; int norm_mode;
};
// rowg[j] = dLoss/dlogp of compact row j in [row0, row0 + rows_max) (0 for padding rows)
void launch_clip_rows(const ClipArgs& a, const int32_t* seqc, const int32_t* row_index, const int32_t* row_counts,
                      int64_t row0, int64_t rows_max, float* rowg, hipStream_t st);
// per generation (in gen_range): its share of the loss, its clipped tokens, the sum of its tokens' KL estimates
void launch_clip_generations(const ClipArgs& a, const int32_t* gen_range, double* loss_n, double* clipped_n, double* kl_n,
                             int32_t* dev_status, hipStream_t st);
// loss and diagnostics from the per-generation sums
void launch_clip_finish(const double* loss_n, const double* clipped_n, const double* kl_n, int64_t N, const int32_t* counts,
                        float* loss_out, rapid_clip_pg_diag* diag, hipStream_t st);
// tsum/tmax given: token-level outer weight (g_n is then the generation's factor without a ratio).
// Three uses.  Whole batch (gen_range, lam_state NULL): coefficients, scale lambda, loss, diagnostics.
// One chunk of the cached backward (gen_range and lam_state given): coefficients of the chunk's generations
// only, scaled by exp(-Lambda) with Lambda = max(lam_state[0], the chunk's own lambda) (0 if not normalized);
// writes Lambda back to lam_state[0] and to lam_chunk[0], and to beta_out[0] the factor
// exp(old Lambda - new Lambda) that the gradient sums accumulated so far have to be multiplied by; no loss,
// no diagnostics.  Closing pass (write_g = 0): loss and diagnostics of
// the whole batch, no coefficient is written.
struct CoefArgs {
    const double* s64; const float* adv; const double* adv64; const float* coef_override; int64_t N;
    float eta; int coef_mode; float loss_scale; int normalized;
    const double* tsum; const double* tmax; const int32_t* counts;
    float* g; double* g64; float* loss_out; rapid_iw_pg_diag* diag;
    const int32_t* gen_range; double* lam_state; double* lam_chunk; float* beta_out; int write_g;
};
void launch_coefficients(const CoefArgs& a, hipStream_t st);
// rowg[j] = dL/dlogp of compact row j in [row0, row0 + rows_max) (0 for padding rows): g of its generation,
// times its own ratio if per_token
void launch_row_coefficients(const float* g, const double* g64, const int32_t* seqc, const int32_t* row_index,
                             const int32_t* counts, const float* logp_cur, const float* logp_behav, int per_token,
                             float eta, int clip_tokens, int64_t row0, int64_t rows_max, float* rowg, hipStream_t st);
// cached backward with normalized gradients: every valid dhidden row of generation n is multiplied by
// exp(lam_chunk[gen_chunk[n]] - lam_state[0]) (the scale its chunk used against the final one)
void launch_rescale_rows(void* dhidden, const uint8_t* mask, int64_t N, int64_t T, int64_t d, const int32_t* gen_chunk,
                         const double* lam_chunk, const double* lam_state, hipStream_t st);
void launch_fill_f64(double* p, int64_t n, double v, hipStream_t st);
void launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st);
// dst[i] += src[i]
void launch_f32_add(const float* src, float* dst, int64_t n, hipStream_t st);
// rows of masked positions, and (idle != NULL) of every position of an idle generation, set to zero
void launch_zero_masked_rows(void* dhidden, const uint8_t* mask, int64_t rows, int64_t d, int elem_bytes,
                             const int32_t* idle, int64_t T, hipStream_t st);
void launch_f32_to_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t st);

// ---- pack.hip ---------------------------------------------------------------------------------
// dst[r][c] (ld_dst) = src[srow(r)][c] for r < R, c < C else 0, over r < Rpad, c < Cpad.
// R may come from the device: if counts != NULL, R = counts[CNT_M] - r0 clipped to [0, R] and
// Rpad = counts[CNT_MR] - r0 clipped to [0, Rpad].  Source row of r is row_index[r0 + r] if
// row_index is given, else r (the caller offsets `src`).
void launch_copy_pad_bf16(const bf16_t* src, int64_t ld_src, const int32_t* row_index, bf16_t* dst,
                          int64_t ld_dst, int64_t R, int64_t C, int64_t Rpad, int64_t Cpad,
                          const int32_t* counts, int64_t r0, hipStream_t st);
// dst[c][r] (ld_dst) = src[r][c] for r < R, c < C else 0, over r < Rpad, c < Cpad.
void launch_block_rows_bf16(const bf16_t* src, int64_t ld, bf16_t* dst, int64_t R, int64_t C, int RB, hipStream_t st);
void launch_transpose_pad_bf16(const bf16_t* src, int64_t ld_src, bf16_t* dst, int64_t ld_dst, int64_t R,
                               int64_t C, int64_t Rpad, int64_t Cpad, const int32_t* counts, int64_t r0,
                               hipStream_t st);

// ---- rmsnorm.hip ------------------------------------------------------------------------------
// dst row r in [r0, r0 + Rpad) below counts[CNT_MR] = bf16(src[row_index[r]] * weight / rms) for r < counts[CNT_M],
// zero otherwise and in columns C .. Cpad; inv_rms[r] = 1 / sqrt(mean(x^2) + eps).  C % 8 == 0.  dst and
// inv_rms are indexed by compact row.
void launch_rmsnorm_pad_bf16(const bf16_t* src, int64_t C, const int32_t* row_index, const bf16_t* weight, float eps,
                             bf16_t* dst, int64_t ld_dst, int64_t r0, int64_t Rpad, int64_t Cpad, const int32_t* counts,
                             float* inv_rms, hipStream_t st);
// dh [N*T, d] holds dL/dh at the valid positions of the compact rows [row0, row0 + rows_max) below
// counts[CNT_M]: if part != NULL, partial sums of dL/dweight over blocks of those rows go to
// part [rmsnorm_dweight_blocks(rows_max)][d] (zeroed beforehand: a block without rows writes nothing); then dh
// becomes dL/dx in place.  launch_rmsnorm_dweight_reduce sums nblk blocks of partial sums in order.
int64_t rmsnorm_dweight_blocks(int64_t rows_max);
void launch_rmsnorm_backward(const bf16_t* x, bf16_t* dh, int64_t d, const bf16_t* weight, const int32_t* row_index,
                             const int32_t* counts, const float* inv_rms, int64_t row0, int64_t rows_max, float* part,
                             hipStream_t st);
void launch_rmsnorm_dweight_reduce(const float* part, int64_t d, int64_t nblk, float* dweight, hipStream_t st);

// ---- gemm_bf16.hip ----------------------------------------------------------------------------
struct FwdArgs {          // logits tile -> per-slot (max, sumexp) and gathered logit
    const bf16_t* Wvd;    // [Vpad, dpad]
    const bf16_t* Hc;     // [Mmax_pad, dpad]
    int64_t dpad;         // contraction extent (multiple of 64)
    int64_t ldk;          // leading dimension of Wvd and Hc (elements)
    int tilesV, tilesM;   // 256-tiles (tilesM: row tiles of this launch, from row0 on; rows past the last token are skipped)
    int64_t row0;         // first compact token row of this launch
    int64_t V;
    float inv_temp;
    const int32_t* tokc;
    const int32_t* counts;
    float* part_max;      // [P][ld_part], P = tilesV * 2
    float* part_sum;
    int64_t ld_part;
    float* zy;            // [Mmax_pad]
    int gi;               // tiles along i that share one j before the order moves on (L2 blocking)
    bf16_t* zc;           // NULL, or [rows, ldz]: the kernel also stores exp(logit - refz[row]) there; refz must be set
    int64_t ldz;
    float* refz;          // [Mmax_pad] reference of the stored exponentials, written by launch_token_logit if zc is set
    const float* ref_logp;   // NULL, or [N*T] log-probs subtracted from zy to form refz
    const int32_t* row_index;
    int32_t* dev_status;  // may be NULL
    int64_t part_row0 = 0;   // compact row whose partials sit in column 0 of part_max / part_sum
    int64_t zc_row0 = 0;     // compact row stored in row 0 of zc
    const bf16_t* WvdB = nullptr;   // if set: W blocked per (256-row tile, K step of 32) (launch_block_w32); selects the
                                    // kernel that runs two workgroups per CU
    int k32_mode = 1;               // with WvdB: 1 = two 4-wave workgroups per CU on 256 x 128 tiles, 2 = one 8-wave
                                    // workgroup per CU on 256 x 256 tiles with requests three K steps ahead
};
void launch_fwd_lse(const FwdArgs& a, hipStream_t st);
// out [Vpad * dpad]: Wvd [Vpad, ldk] in blocks of 256 rows x 32 columns, in the LDS order of the two-workgroup forward
void launch_block_w32(const bf16_t* Wvd, int64_t ldk, bf16_t* out, int64_t Vpad, int64_t dpad, hipStream_t st);
// zy (and refz) for the compact rows [row0, row0 + rows_max)
void launch_token_logit(const FwdArgs& a, int64_t row0, int64_t rows_max, hipStream_t st);
int fwd_slots_per_tile();

struct DzArgs {           // logits tile -> dz = g (onehot - p) / temperature, bf16 [Mc, Vpad]
    const bf16_t* Wvd;
    const bf16_t* Hc;     // already offset to the chunk's first row
    int64_t dpad, ldk;
    int tilesV, tilesM;   // tilesM = chunk rows / 256
    int64_t V, Vpad;
    int64_t ldz;          // leading dimension of dz
    float inv_temp;
    int64_t m0;           // first compact row of the chunk
    const int32_t* tokc;  // full arrays (indexed by compact row)
    const float* lse_c;
    const float* rowg;    // dL/dlogp per compact row
    const int32_t* counts;
    bf16_t* dz;           // [Mc, Vpad]
    int gi;               // tiles along i that share one j before the order moves on (L2 blocking)
};
void launch_dz(const DzArgs& a, hipStream_t st);
// turns the ratios a storing forward left in u [rows_max, ldz] (row 0 = compact row row0) into the
// backward's operands: the sampled token's element of each row, the row factors rowc, and Hc scaled by
// them in place (Hc, tokc, zy, refz, lse_c, rowg, rowc are indexed by compact row)
void launch_cache_finish(bf16_t* u, int64_t ldz, bf16_t* Hc, int64_t ldk, const int32_t* tokc,
                         const float* zy, const float* refz, const float* lse_c, const float* rowg, float inv_temp,
                         const int32_t* counts, int64_t row0, int64_t rows_max, float* rowc, int32_t* dev_status,
                         hipStream_t st);

struct DhArgs {           // dH[row, :] = dz[row, :] . Wdv^T
    const bf16_t* Wdv;    // [dpadR, Vpad]
    const bf16_t* WdvB;   // the same, tile-blocked (blocks of tile-rows x 64 columns), or NULL
    const bf16_t* dz;     // [Mc, Vpad]
    int64_t Vpad;         // contraction extent
    int64_t ldv;          // leading dimension of Wdv and dz
    int64_t d, dpadR;
    int tilesM;
    int64_t m0;
    const int32_t* row_index;
    const int32_t* counts;
    const float* rowc;    // NULL, or one factor per compact row applied to the result
    unsigned* pace;       // NULL, or one word, zero at launch: arrival counter of the launch's workgroups
    int pace_every;       // K steps between meetings (power of two)
    bf16_t* dhidden;      // [N*T, d]
    int gi;               // tiles along i that share one j before the order moves on (L2 blocking)
    float* part = nullptr;    // NULL, or scratch of part_bytes: lets the kernel cut a partly filled last round of tiles
    size_t part_bytes = 0;    // along the contraction (needs 512 KiB per workgroup of the launch)
};
void launch_dh(const DhArgs& a, hipStream_t st);
size_t dh_part_bytes();   // scratch that lets every dHidden launch cut its last round

struct DwArgs {           // dW (+)= Hc^T . dz over the chunk's rows
    const bf16_t* dz;     // [Mc, Vpad] chunk (rows = tokens)
    const bf16_t* Hc;     // [Mmax_pad, >= dpadR], already offset to the chunk's first row
    int64_t Mc;           // rows of the chunk buffer (contraction extent is min(Mc, rows left))
    int64_t ldz, ldH;     // leading dimensions of dz and Hc
    int64_t d, dpadR, V, Vpad;
    int64_t m0;
    const int32_t* counts;
    float* dW;            // fp32, layout per w_layout
    int w_layout;
    int beta;             // 0 overwrite, 1 accumulate
    const float* beta_scale = nullptr;   // NULL, or device: with beta = 1 the old value is multiplied by beta_scale[0] first
    int gi;               // tiles along i that share one j before the order moves on (L2 blocking)
};
void launch_dw(const DwArgs& a, hipStream_t st);
void set_waves_per_workgroup(int n);   // 4, 8 or 16 waves per contraction workgroup
void set_dw_deep(int on);              // dW with K steps of 32 rows and requests three steps ahead
void set_cu_count(int n);              // compute units of the device: the contraction kernels launch one workgroup each


void launch_sgd_step(float* master, const float* grad, int64_t n, float lr, void* w_out, int dtype, hipStream_t st);
void launch_adamw_step(float* master, const float* grad, float* m, float* v, int64_t n, float lr, float beta1, float beta2,
                       float eps, float weight_decay, int64_t step, void* w_out, int dtype, hipStream_t st);

// ---- probe.hip -----------------------------------------------------------------------------------
int run_mfma_probe(int random_operands, int iters, int num_cu, double* tflops_out, double* ms_out, hipStream_t st);

// ---- f32_path.hip -----------------------------------------------------------------------------
// C[i][j] (+)= alpha sum_k A(i,k) B(k,j), arbitrary strides, optional index maps, and a device-side
// row count.  Accumulates in fp64.
struct F32Gemm {
    const float* A; int64_t sa_i, sa_k;
    const int32_t* a_imap;   // optional: A row of i is a_imap[i0 + i]
    const int32_t* a_kmap;   // optional: A position of k is a_kmap[i0 + k]
    const float* B; int64_t sb_k, sb_j;
    float* C; int64_t sc_i, sc_j;
    const int32_t* c_rows;   // optional: C row of i is c_rows[i0 + i]
    int64_t I, J, Kd;
    int beta;
    const int32_t* counts; int64_t i0;   // if counts: I (or Kd when limit_k) is clipped to M - i0
    int limit_k;
    float alpha;
};
void launch_f32_gemm(const F32Gemm& g, hipStream_t st);
// row-wise: lse, logp, gathered logit from a materialised logits chunk z [rows, V]
void launch_f32_row_lse(const float* z, int64_t V, int64_t rows, int64_t m0, const int32_t* tokc,
                        const int32_t* row_index, const int32_t* counts, float* lse_c, float* logp_out,
                        float* lse_out, hipStream_t st);
// in place: z -> dz = g (onehot - softmax) * inv_temp
void launch_f32_dz(float* z, int64_t V, int64_t rows, int64_t m0, const int32_t* tokc,
                   const float* lse_c, const float* rowg, float inv_temp, const int32_t* counts, hipStream_t st);

void set_error(const char* fmt, ...);

}  // namespace rapid
