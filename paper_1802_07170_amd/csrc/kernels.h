// Host-callable launchers of the gfx950 kernels.  `prec` selects the storage type of GEMM
// operands: 0 = float, 1 = bf16 (raw uint16).  "T*" in comments means that type.
// All launchers only enqueue work on `st`; none allocates or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cmt {

// ---- gemm.hip ----------------------------------------------------------------------------------
// C[M,N] = A[M,K] * B[N,K]^T (+ bias[N]) (+ previous C when accumulate), both operands with k
// contiguous.  Writes fp32 to Cf (if non-null) and T to Ct (if non-null), same ldc.
// K, lda, ldb multiples of 8.
// When split_scratch is given and the output has few tiles but K is long, k is split over workgroups
// into fp32 planes in the scratch (at most 8 * M * N floats) that a second kernel sums.
// A row count known only on the device (the number of valid target positions): the count a kernel
// works on is clamp(*n - base, 0, the count the host passed).  n = null: the host's count.
struct RowLimit { const int32_t* n = nullptr; int base = 0; };
// limit_kind 1: `limit` bounds M (tiles beyond it exit; rows beyond it are not stored);
// limit_kind 2: `limit` bounds K, rounded up to a multiple of 64 (the callers zero-fill both operands there); a
// workgroup whose contraction is empty exits without touching C.
void launch_gemm_nt(int prec, const void* A, int lda, const void* B, int ldb, int M, int N, int K,
                    float* Cf, void* Ct, int ldc, const float* bias, int accumulate, hipStream_t st,
                    float* split_scratch = nullptr, size_t split_scratch_floats = 0, RowLimit limit = RowLimit{},
                    int limit_kind = 0, int wg_cap = 0);
// wg_cap > 0: at most that many workgroups (rounded up to a multiple of 8) walk the tiles — for a GEMM on a second
// stream that is to leave part of the chip to the kernels of the first.
// Matrix-core issue-rate probe: `blocks` workgroups of 4 wavefronts, each `iters` x 4 bf16 32x32x16 MFMAs on
// registers; out needs blocks * 256 floats.  Returns the flops of the launch.
// Several independent C (+)= A * B^T problems (fp32 C, no bias) as one launch: the tiles of all problems form one
// queue spread over the chip, so that small problems fill each other's partial rounds and there are no gaps between
// them (the weight-gradient GEMMs of the step, the paper's calculateGradient with beta = 1 batched over time).
struct GemmProb { const void* A; const void* B; float* C; int lda, ldb, ldc, M, N, K, accumulate; };
// split_scratch: planes for the fp32 path, which launches the problems one by one (see launch_gemm_nt).
void launch_gemm_nt_group(int prec, const GemmProb* probs, int n, hipStream_t st, float* split_scratch, size_t split_scratch_floats,
                          int wg_cap = 0);
double launch_mfma_rate(float* out, int blocks, int iters, hipStream_t st);
// out[C,R] = in[R,C]^T for T matrices (ldin, ldout in elements).
void launch_transpose(int prec, const void* in, int ldin, void* out, int ldout, int R, int C, hipStream_t st);

// ---- ce.hip ------------------------------------------------------------------------------------
// Eq. 1 for a slab of M <= pitch rows (all row pointers at the slab's first row; pitch = row capacity of the
// slab buffers, a multiple of 64).
// Forward: Ho [M,H] T, Wo [V,H] T, Bo [V] fp32, labels [M] int32.  Per row and group of 64
// vocabulary columns: pmax = max z, psum = sum exp(z - pmax) ([np, pitch] fp32: group-major, np = ce_num_partials(V));
// zy [M] = the label's logit; ET [V, pitch] T = exp(z - pmax of its group), transposed;
// psz (same layout) = sum of z over the group (null unless label smoothing needs the row's mean logit).
// A slab holds up to CE_SLAB_MAX_ROWS target positions (fewer when the handle is created for fewer): the whole
// batch is one slab up to that size, which measured faster than several smaller ones (one pass over W_o and one
// read-modify-write of its gradient per slab).  The pitch adds 64 to the capacity so that it is never a power of two.
constexpr int CE_SLAB_MAX_ROWS = 16384;
int ce_num_partials(int V);
inline int ce_slab_pitch(int rows) { return rows + 64; }
// Every launcher below takes a RowLimit: the slab's row count as the device knows it (see
// launch_ce_compact); rows beyond it are neither computed nor stored.
void launch_ce_fwd(int prec, const void* Ho, int ldho, const void* Wo, const float* Bo, const int32_t* labels,
                   int M, int V, int H, void* ET, int pitch, float* pmax, float* psum, float* psz, float* zy, hipStream_t st,
                   RowLimit lim = RowLimit{});
// The valid target positions of the batch (mask > 0, M = all rows, time-major) numbered consecutively:
// pos[M] = index or -1, row[index] = row, labels_c / rowscale_c [index] = label and 1 / n_tok,
// *n_valid = loss[1] = n_tok.  The output layer then runs on the dense rows [0, n_valid).
void launch_ce_compact(const float* mask, const int32_t* labels, int M, int32_t* pos, int32_t* row, int32_t* labels_c,
                       float* rowscale_c, int32_t* n_valid, float* loss, hipStream_t st);
// dst[c, 0:cols] = src[row[c], 0:cols] for c < *n_valid, zero rows up to the next multiple of 64 (T rows; grid sized for max_rows)
void launch_ce_gather_rows(int prec, const void* src, int lds, const int32_t* row, const int32_t* n_valid, int max_rows, void* dst,
                           int ldd, int cols, hipStream_t st);
// lse[M] and the row loss nll[M] = (1 - eps) (lse - zy) + eps (lse - mean_v z_v) from the partials
// (label smoothing eps of the hyperparameter table; eps = 0: plain negative log-likelihood);
// mask (may be null = all rows count) zeroes the loss of padded rows.
void launch_ce_rows(const float* pmax, const float* psum, const float* psz, const float* zy, const float* mask, int M, int np,
                    int pitch, float eps, int V, float* lse, float* nll, hipStream_t st, RowLimit lim = RowLimit{});
// loss[0] = sum nll / loss[1]; flags |= 4 if it is not finite.  One block, deterministic order.
void launch_ce_loss(const float* nll, int M, float* loss, int* flags, hipStream_t st, RowLimit lim = RowLimit{});
// Backward: ET -> dzT = (ET * exp(pmax - lse) - (1 - eps) onehot - eps / V) * rowscale in place
// ([V, pitch] T; columns >= Mc up to the next multiple of 64 are zero-filled) and dz [Mc, V] T.  The caller
// then takes dH_o[rows] = dz W_o and dW_o += dz^T H_o[rows] with launch_gemm_nt.  dbo_part
// [ceil(Mc / 64), V] fp32: column sums of dz over each block of 64 rows (dB_o = their sum over all slabs).
void launch_ce_scale(int prec, void* ET, int pitch, int V, int Mc, const float* pmax, const float* lse, const int32_t* labels,
                     const float* rowscale, float eps, void* dz, float* dbo_part, hipStream_t st, RowLimit lim = RowLimit{});

// ---- step.hip ----------------------------------------------------------------------------------
// A value delivered as `np` partial planes: v(b, c) = sum_k p[k * stride + b * ld + c]  (np = 0: zero).
// Independent instances (layers / directions working on different time steps) that one launch of a
// step kernel can carry.
constexpr int STEP_MAX_INST = 8;
struct Planes { const float* p; int ld; int np; size_t stride; };
// Number of k-blocks (= planes written) by launch_step_gemm for N output columns, contraction
// length K and padded batch Bp (at most 8).
int step_kblocks(int prec, int N, int K, int Bp, int max_kb = 0);

// Dropout of one [Bp, width] slice of a dropout site (Settings section: dropout on the hidden states
// between recurrent layers and on H_o).  Element (b, col) keeps its value, scaled by `scale`
// = 1 / (1 - p), iff the top 24 bits of SplitMix64(key0 + b * width + col) are >= thresh
// = floor(p * 2^24); key0 = seed + site * 2^48 + t * B * width with B the real batch size.
// on = 0: identity.
struct DropSpec { unsigned long long key0 = 0; unsigned thresh = 0; float scale = 1.f; int width = 0; int on = 0; };

// One recurrent step of one LSTM layer (or of both directions of the bottom encoder layer when
// ndir = 2): gates = Gx + [x; h_prev] W^T, then the cell, fused.
struct LstmFwdDir {
  const void* x;  int ldx;  int Kx;     // per-step input segment (T*, [Bp, Kx]); Kx = 0 if none
  const void* hprev; int ldh;           // previous state (T*, [Bp, Hh])
  const void* W;  int ldw;  int wx_off, wh_off;   // weights T* [4Hh, ldw]; column offsets of the segments
  const float* gx; int ldgx;            // batched input pre-activations incl. bias [Bp, 4Hh], or null
  const float* bias;                    // [4Hh], used when gx is null
  const float* cprev;                   // [Bp, Hh]
  const float* mask;                    // [Bp] 1 = valid step
  void* hnext; int ldhn; float* cnext;  // next state (T*, row pitch ldhn); cell state [Bp, Hh]
  float* gsave;                         // [Bp, 4Hh] gate activations kept for the backward pass
  void* ycat; int ldy;                  // optional second copy of h (T*, row pitch ldy), or null:
  DropSpec drop{}; int drop_col0 = 0;   //   the layer's output as the layer above sees it, i.e. after
                                        //   dropout (columns drop_col0 + [0, Hh) of the site)
  // Fragment-major copies (16-bit operands, see fm_offset; null = not used).  With W_fm set the contraction reads
  // W_fm (the columns [wh_off - Kx, wh_off + Hh) of W), x_fm (if Kx > 0) and hprev_fm instead of W, x and hprev;
  // hnext_fm / ycat_fm receive a second copy of what goes to hnext / ycat.  Needs Kx and Hh multiples of 32.
  const void* W_fm = nullptr; const void* x_fm = nullptr; const void* hprev_fm = nullptr;
  void* hnext_fm = nullptr; void* ycat_fm = nullptr;
};
// Fragment-major storage of a 16-bit matrix [rows, K] that a step kernel reads as a matrix-core operand: 1 KB blocks
// [row / 16][k / 32][lane][8 elements] with lane = row % 16 + 16 * ((k % 32) / 8) — the register image of the
// 16x16x32 MFMA operand, so that a wavefront's fragment load is one contiguous kilobyte instead of 16 pieces of
// 64 bytes from 16 rows (measured on the decoder layer step: 2.3 times the rate from L2).  nsteps = K / 32.
inline __host__ __device__ size_t fm_offset(int row, int k, int nsteps) {
  return ((((size_t)(row >> 4) * nsteps + (k >> 5)) * 64 + (row & 15) + 16 * ((k & 31) >> 3)) << 3) + (k & 7);
}
// dst (fragment-major, nsteps = cols / 32) <- src [rows, cols] row-major with pitch ld (16-bit elements; rows a
// multiple of 16, cols a multiple of 32).  With dst_nsteps > 0 the destination is a wider matrix of dst_nsteps
// k steps per row tile and the copy lands at its columns [32 * dst_step0, 32 * dst_step0 + cols).
void launch_fm_pack(const void* src, int ld, int rows, int cols, void* dst, hipStream_t st, int dst_nsteps = 0, int dst_step0 = 0);
// the same for the gate rows of an LSTM weight matrix: tile T holds units 4T .. 4T+3, row m of the tile is gate m % 4
// of unit 4T + m / 4 (rows of W are gate-major: gate * Hh + unit); columns [col0, col0 + K) of W
void launch_fm_pack_lstm_weights(const void* W, int ldw, int col0, int K, int Hh, void* dst, hipStream_t st);
// ndir <= STEP_MAX_INST instances of equal hidden width Hh in one launch.
void launch_lstm_fwd(int prec, const LstmFwdDir* dirs, int ndir, int Bp, int Hh, hipStream_t st);

// [a0; a1] W^T for one step.  W rows are output columns; w0_off / w1_off are the column offsets
// inside a weight row that pair with the two activation segments.
struct StepGemm {
  const void* a0; int lda0; int K0; int w0_off;
  const void* a1; int lda1; int K1; int w1_off;
  const void* W; int ldw;
  int N;
  int mode;            // 0: tanh of the sum -> outT (T*) [Bp, N]   (attentional layer, Eq. 7);
                       //    `out` is scratch for the planes when the k range is split
                       // 1: partial planes out[kb][b][n] (fp32, row pitch ldout, plane pitch plane_stride),
                       //    kb < step_kblocks(prec, K0 + K1); the consumer sums them
                       // 2: (max_kb = 1) per block of 64 output columns and sentence the largest value of
                       //    sum + bias[n] and its column, the lower column on equal values:
                       //    out[blk * Bp + b] and best_idx[blk * Bp + b], blk < ceil(N / 64); nothing else is stored
                       // 3: (whole k range in the workgroup) the plain sums out[b * ldout + n] (fp32), nothing else
  int skip0 = 0;       // contract segment 1 only (segment 0 keeps its place in the weight rows and in W_fm)
  void* outT; int ldo;
  void* outD = nullptr; int ldod = 0;  // mode 0: optional copy of outT after dropout `drop`
  DropSpec drop{};
  // fragment-major operands (16-bit types; all that apply or none; K0, K1 multiples of 32, N of 16): W_fm = rows
  // [w_tile0 * 16, ...) of a packed matrix whose k axis is this GEMM's [segment 0; segment 1]; a0_fm, a1_fm
  const void* W_fm = nullptr; int w_tile0 = 0; const void* a0_fm = nullptr; const void* a1_fm = nullptr;
  void* outF = nullptr;                // mode 0, 16-bit types: optional fragment-major copy (fm_offset, N / 32 k steps) of
                                       //   what the next step is fed: outD's values if outD is set, else outT's
  void* outF2 = nullptr;               // one more such copy, into the columns [outF2_k0, outF2_k0 + N) of a fragment-major
  int outF2_nsteps = 0, outF2_k0 = 0;  //   matrix of outF2_nsteps k steps (k0 a multiple of 32)
  float* out; int ldout; size_t plane_stride;
  int max_kb;          // cap on the number of k blocks (planes); 0 = default (8)
  const float* bias = nullptr; int32_t* best_idx = nullptr;   // mode 2
};
void launch_step_gemm(int prec, const StepGemm& g, int Bp, hipStream_t st);
// n <= STEP_MAX_INST instances in one launch (mode 1 only): same K0 + K1 and max_kb, N may differ; the
// number of planes each instance writes is step_kblocks of the widest one.
// n_plan > 0 fixes the width the k-block plan is made for (so that it does not change from launch to launch).
void launch_step_gemm_multi(int prec, const StepGemm* gs, int n, int n_plan, int Bp, hipStream_t st);

// Cell backward for one step of one layer: builds dgates (T*) from the incoming state gradients.
struct LstmBwdPoint {
  Planes dy; int dy_col;               // gradient arriving at this step's output: columns dy_col + [0, Hh)
  DropSpec drop_dy{};                  // dropout between this layer and its consumer (same columns)
  Planes dhrec; int dhrec_col;         // recurrent part of d state from the next step's GEMM
  float* dh;                           // [Bp,Hh] in: pass-through part of d state; out: (1-m) * total
  float* dc;                           // [Bp,Hh] in/out cell-state gradient
  const float* gsave;                  // [Bp,4Hh]
  const float* cprev; const float* cnext;  // [Bp,Hh]
  const float* mask;                   // [Bp]
  void* dg; int lddg;                  // T* [Bp,4Hh], row pitch lddg
  void* dg_fm = nullptr;               // optional fragment-major copy of dg (16-bit types; 4Hh / 32 k steps)
};
void launch_lstm_bwd_point(int prec, const LstmBwdPoint& p, int Bp, int Hh, hipStream_t st);
void launch_lstm_bwd_point_multi(int prec, const LstmBwdPoint* ps, int n, int Bp, int Hh, hipStream_t st);
// Backward step GEMM with the whole contraction inside the workgroup and the consumer of its result fused
// into the epilogue: out[Bp, N] = dg[Bp, K] * Wt[N, K]^T, where the N output columns come in two parts
// (part 0 first), each with its own epilogue:
//   BWD_EPI_STORE     the values are stored as fp32 to out [Bp, ncols] (row pitch ldout);
//   BWD_EPI_CELL_DY   the values are the gradient arriving at the output of the LSTM step `cell` (the layer
//                     below, same time step: dx of this layer), added to cell.dy; the cell backward runs
//                     in-register and writes that step's dgates;
//   BWD_EPI_CELL_REC  the values are the recurrent part of the state gradient of the LSTM step `cell` (this
//                     layer, the next step of the backward loop: dh_prev), added to cell.dhrec;
//   BWD_EPI_TANH      the values are the input-feed gradient of H_o of the previous decoder step:
//                     dpre = (dce[pos[b]] + value) * drop * (1 - Ho^2), as launch_tanh_bwd computes it.
// ncols of part 0 is a multiple of 16; both are multiples of 4.  hh = hidden width of `cell` (CELL_*) or the
// row width of dce (TANH).
enum { BWD_EPI_STORE = 0, BWD_EPI_CELL_DY = 1, BWD_EPI_CELL_REC = 2, BWD_EPI_TANH = 3 };
struct BwdEpi {
  int kind = BWD_EPI_STORE; int ncols = 0; int hh = 0;
  float* out = nullptr; int ldout = 0;
  LstmBwdPoint cell{};
  const float* dce = nullptr; const int32_t* pos = nullptr; const void* Ho = nullptr; int ldho = 0;
  void* dpre = nullptr; int ldp = 0; DropSpec drop{};
  void* dpre_fm = nullptr;             // TANH: optional fragment-major copy of dpre (hh / 32 k steps)
};
struct StepBwd {
  const void* dg; int lddg; int K;     // T* [Bp, K]
  const void* Wt; int ldw;             // T* [N, K]: row n = output column n
  BwdEpi part[2];
  // fragment-major operands (16-bit types; both or none): dg_fm = the same [Bp, K]; Wt_fm = the whole transposed
  // weight matrix, of which this instance's rows start at row tile wt_tile0 (16 rows per tile)
  const void* dg_fm = nullptr; const void* Wt_fm = nullptr; int wt_tile0 = 0;
};
constexpr int STEP_BWD_MAX_INST = 4;
// Attention scores that ride in a step GEMM's launch: dots[b, i] = vec[b, :] . Mat[i, b, :] for i < len[b]
// (Mat rows [S * Bp, ldm]: T*, or float* with mat_f32 set; vec rows [Bp, ldv]: T*; dots fp32 [Bp, S])
struct AttScores { const void* Mat; int ldm; const void* vec; int ldv; const int32_t* len; int S, H; float* dots; int mat_f32; };
// n independent instances in one launch (more than STEP_BWD_MAX_INST are spread over several launches).
// With `scores` (n = 1) further workgroups of the launch compute those scores; they must depend on nothing the
// instance writes.
void launch_step_bwd_fused(int prec, const StepBwd* gs, int n, int Bp, hipStream_t st, const AttScores* scores = nullptr);

// out[Bp, cols] = base (or 0) + planes columns col0 + [0, cols)
void launch_planes_add(float* out, const float* base, const Planes& p, int col0, int Bp, int cols, hipStream_t st);

// Attention forward for one decoder step (Eq. 3-5 with the key hoist K_i = W_a^T H_s^i):
// s_i = K_i . H_t, softmax over i < src_len[b], C_s = sum a_i H_s^i.  dots [Bp,S] is scratch.
// ldk / lds / ldt / ldcs: row pitches (elements) of Kmat, Hs, Ht and Cs.
void launch_att_fwd(int prec, const void* Kmat, int ldk, const void* Hs, int lds, const void* Ht, int ldt,
                    const int32_t* src_len, int S, int Bp, int H, float* dots, float* a /*[Bp,S]*/,
                    void* Cs /*T* [Bp,ldcs]*/, int ldcs, hipStream_t st, void* Cs_fm = nullptr /* fragment-major copy */);
// The same step with the context half of the attentional layer hoisted out of the loop (Eq. 5-7):
// W_c [C_s; H_t] = sum_i a_i (W_c1 H_s^i) + W_c2 H_t, where the rows P_i = W_c1 H_s^i (Pmat: T* [S * Bp, ldp], like Kmat)
// are made once per batch.  Two launches: (1) the scores s_i = K_i . H_t and, in other workgroups of the same launch, the plain
// sums u = W_c2 H_t (fp32 [Bp, H] at `u.out`; `u` is a StepGemm of mode 3 with skip0 set, below 256 sentences);
// (2) softmax, sum a_i P_i + u, tanh -> H_o with the copies a mode-0 StepGemm writes (described by `o`).
// C_s itself is not made here: launch_att_context makes it for all steps at once.
struct AttOut {
  void* outT; int ldo;                 // H_o rows [Bp, ldo]
  void* outD = nullptr; int ldod = 0;  // optional copy after dropout `drop`
  DropSpec drop{};
  void* outF = nullptr;                // 16-bit types: optional fragment-major copy (H / 32 k steps) of outD's values, else outT's
  void* outF2 = nullptr;               // one more such copy, into the columns [outF2_k0, outF2_k0 + H) of a fragment-major
  int outF2_nsteps = 0, outF2_k0 = 0;  //   matrix of outF2_nsteps k steps (k0 a multiple of 32)
};
void launch_att_fwd_proj(int prec, const void* Kmat, int ldk, const void* Pmat, int ldp, const void* Ht, int ldt,
                         const StepGemm& u, const AttOut& o, const int32_t* src_len, int S, int Bp, int H, float* dots,
                         float* a /*[Bp,S]*/, hipStream_t st);
// C_s[j, b, :] = sum_i a[j, b, i] H_s^i[b, :] for all T steps (Eq. 5); a [T, Bp, S], Cs rows [T * Bp, ldcs]
void launch_att_context(int prec, const void* Hs, int lds, const float* a, const int32_t* src_len, int S, int T, int Bp, int H,
                        void* Cs, int ldcs, hipStream_t st);
// Attention backward for one step.  dCst: planes [.., Bp, 2H] fp32 from the step GEMM dpre W_c:
// columns [0,H) = dC_s, [H,2H) = the part of dH_t that came through the concatenation.
// da_i = dC_s . H_s^i, ds = a (da - sum a da), dHt = dCst[:, H:] + sum ds_i K_i;
// dCs_sum [Bp,H] receives the summed dC_s (kept for the deferred gradients).
// With `cell` (the top decoder layer's step, hidden width H) the cell backward of that step runs in the same
// launch with dHt as the gradient at its output (added to cell->dy), and dHt itself is not stored.
void launch_att_bwd(int prec, const void* Kmat, int ldk, const void* Hs, int lds, const Planes& dCst, float* dCs_sum, const float* a,
                    const int32_t* src_len, int S, int Bp, int H, float* dots, float* ds /*[Bp,S]*/,
                    float* dHt /*[Bp,H]*/, hipStream_t st, const LstmBwdPoint* cell = nullptr);
// The second half of that step when the scores da_i are already in `dots` (with the projected rows P_i = W_c1 H_s^i,
// da_i = dpre . P_i needs no dC_s): ds, dHt = add[:, add_col + [0, H)] + sum ds_i K_i, and the fused cell backward.
void launch_att_bwd_mix(int prec, const void* Kmat, int ldk, const Planes& add, int add_col, const float* a, const int32_t* src_len,
                        int S, int Bp, int H, const float* dots, float* ds /*[Bp,S]*/, float* dHt /*[Bp,H]*/, hipStream_t st,
                        const LstmBwdPoint* cell = nullptr);
// After the decoder loop: dHs_ctx[i,b,:] = sum_j a[j,b,i] dCs[j,b,:], dK[i,b,:] = sum_j ds[j,b,i] Ht[j,b,:].
void launch_att_deferred(int prec, const float* a, const float* ds, const float* dCs, int lddc, const void* Ht, int ldht,
                         int S, int T, int Bp, int H, float* dHs, void* dK, hipStream_t st);
// dpre = (dHo_ce + feed) * drop * (1 - Ho^2) -> T*   (Ho: before dropout; drop: the factors H_o's
// consumers saw)
// dHo_ce: rows [Bp, H] of this step, or — with pos [Bp] given — a dense matrix [n, H] in which row pos[b]
// belongs to sentence b (pos[b] < 0: no row, zero).
void launch_tanh_bwd(int prec, const float* dHo_ce, const int32_t* pos, const Planes& feed, const void* Ho, int ldho, void* dpre,
                     int ldp, int Bp, int H, const DropSpec& drop, hipStream_t st, void* dpre_fm = nullptr /* fragment-major copy */);

// ---- misc.hip ----------------------------------------------------------------------------------
// Embedding gather + masks + input validation (flags |= 1 bad id, |= 2 bad length).
// ids [B, L] row-major; out[t, b, :] = table[shift ? (t == 0 ? bos : ids[b, t-1]) : ids[b, t]] as T;
// rows b >= B are zero.  mask[t, b] = t < len[b].  labels[t, b] = ids[b, t] (only when shift).
void launch_gather(int prec, const void* table, int vocab, int E, const int32_t* ids, const int32_t* len,
                   int B, int Bp, int L, int shift, int bos, void* out, float* mask, int32_t* tok,
                   int32_t* labels, int32_t* len_p, int* flags, hipStream_t st);
// Dense embedding gradient: dE[V,E] = 0, then row id gets the sum of dX rows of its occurrences,
// added in ascending position order by the block of the first occurrence (no atomics).
// zero_first = false: the caller has already cleared dE (e.g. earlier in the step, off the critical path).
void launch_embed_scatter(const float* dX, const int32_t* tok, int n, int V, int E, float* dE, hipStream_t st, bool zero_first = true);
void launch_fill_f32(float* p, size_t n, float v, hipStream_t st);
void launch_fill_T(int prec, void* p, size_t n, hipStream_t st);      // zeros
void launch_cast(int prec, const float* src, void* dst, size_t n, hipStream_t st);   // fp32 -> T
// 2-D copies with pitches (elements): fp32 -> fp32, T -> T.
void launch_copy2d_f32(const float* src, int lds, float* dst, int ldd, int rows, int cols, hipStream_t st);
// Several small zero-fills / 2-D copies in one launch each (the state initialisations of a step), in units of
// 32-bit words: a fill clears `words` words at p; a copy moves rows x cols words with row pitches lds / ldd.
constexpr int MULTI_MAX_JOBS = 32;
struct FillJob { void* p; size_t words; };
struct CopyJob { const void* src; int lds; void* dst; int ldd; int rows; int cols; };
void launch_fill_multi(const FillJob* jobs, int n, hipStream_t st);
void launch_copy2d_multi(const CopyJob* jobs, int n, hipStream_t st);
void launch_copy2d_T(int prec, const void* src, int lds, void* dst, int ldd, int rows, int cols, hipStream_t st);
void launch_add_f32(float* dst, const float* src, size_t n, hipStream_t st);          // dst += src
void launch_sum_parts(const float* parts, int nparts, size_t n, float* out, hipStream_t st);
// db[n] = sum_m dG[m, n] over M rows of a T matrix [M, N].
void launch_colsum(int prec, const void* dG, int ld, int M, int N, float* scratch /*[16*N]*/, float* db, hipStream_t st);
// p <- p - lr g; skipped entirely while *flags != 0 (flags may be null)
// bf16_copy (may be null): the bf16 working copy of p, rewritten in the same pass
void launch_sgd(float* p, const float* g, size_t n, float lr, const int* flags, void* bf16_copy, hipStream_t st);
void launch_init_uniform(float* p, size_t n, uint64_t seed, float scale, hipStream_t st);

// Chip-wide barrier probe: `blocks` workgroups (they must all be resident: at most one per CU) pass `rounds`
// barriers on *counter (zero before the launch); a workgroup that polls max_spin times without success sets
// *gave_up and leaves.  fences: device-scope fences around each barrier.
void launch_grid_barrier_probe(unsigned* counter, int* gave_up, int blocks, int rounds, int fences, int max_spin, hipStream_t st);

// ---- greedy decoding (misc.hip) -------------------------------------------------------------------
// x[b, 0:E] = table[tok[b]] (T, row pitch ldx) for b < B; zero rows for b in [B, Bp).
// x_fm (16-bit types, optional): the same rows into the columns [0, E) of a fragment-major matrix of nsteps_fm k steps.
void launch_dec_embed(int prec, const void* table, int E, const int32_t* tok, int B, int Bp, void* x, int ldx, hipStream_t st,
                      void* x_fm = nullptr, int nsteps_fm = 0);
// tok[b] = argmax_v (z[b, v] + bias[v]) (lowest index on ties); unfinished sentences record it at
// out_ids[b, j] and end on eos or at j = max_len - 1 (done[b] = 1, out_len[b] = j + 1).
// With `table` (T [V, E]) the kernel also writes the token's embedding row to x[b, 0:E] (T, row pitch ldx) and, for
// 16-bit types, to the fragment-major x_fm (nsteps_fm k steps): the next step's input, for b < B.
// With part_idx the candidates are not logits but per-sentence partial results: z[k * ldz + b] and part_idx[k * ldz + b],
// k < V, hold a value (bias included) and its token; `bias` is not used.
void launch_dec_argmax(const float* z, int ldz, const float* bias, int V, int B, int j, int max_len, int eos, int32_t* tok,
                       int32_t* done, int32_t* out_ids, int32_t* out_len, hipStream_t st, int prec = 0, const void* table = nullptr,
                       int E = 0, void* x = nullptr, int ldx = 0, void* x_fm = nullptr, int nsteps_fm = 0,
                       const int32_t* part_idx = nullptr);
// tok = bos, done = 0, out_ids = pad, out_len = 0, mask[b] = (b < B).
void launch_dec_init(int B, int Bp, int max_len, int bos, int pad, int32_t* tok, int32_t* done, int32_t* out_ids, int32_t* out_len,
                     float* mask, hipStream_t st);

// ---- beam search (beam.hip) -----------------------------------------------------------------------
// Device-side state of a search over R = B * K rows (row r = b * K + s: live hypothesis s of sentence b).
struct BeamState {
  float* cum; float* new_cum;            // [Rp] summed log-probabilities of the live hypotheses (-inf: dead slot)
  int32_t* tok; int32_t* new_tok;        // [Rp] previous token of every row (next step's input)
  int32_t* parent;                       // [Rp] row a new hypothesis continues (-1: dead slot)
  float* mask;                           // [Rp] 1 = live row
  int32_t* nlive;                        // [B] live hypotheses per sentence
  float* fin_score; int32_t* fin_step; int32_t* fin_par; int32_t* fin_tok;   // [B] best finished hypothesis
  int32_t* hist_tok; int32_t* hist_par;  // [steps, hist_ld] token / parent slot of every live hypothesis per step
  int hist_ld;
  float* row_lse;                        // [Rp] log-sum-exp of the row's logits of the current step
  float* cand_z; int32_t* cand_tok;      // [Rp, 16] the row's best logits / tokens of the current step, best first
};
struct BeamReorder {
  const void* h_src[8]; void* h_dst[8]; int ldh;     // per layer: states written by the step -> states the next step reads
  void* h_dst_fm[8] = {};                            // optional fragment-major copies of h_dst (16-bit types, H / 32 k steps)
  const float* c_src[8]; float* c_dst[8];
  const void* ho_src; int ldho_src; void* ho_dst; int ldho_dst;   // H_o of the step -> input feed of the next
  void* ho_dst_fm = nullptr; int ho_fm_nsteps = 0, ho_fm_k0 = 0;  // optional fragment-major copy: columns [k0, k0 + H) of a
                                                                  //   matrix of ho_fm_nsteps k steps (16-bit types)
};
// dst[i, r, 0:cols] = src[i, r / K, 0:cols] (r < R), zero rows up to Rp; elem_bytes 2 or 4.
void launch_beam_expand(int elem_bytes, const void* src, int ld_src, int rows_src, void* dst, int ld_dst, int n_outer, int R, int Rp,
                        int K, int cols, hipStream_t st);
void launch_beam_init(const BeamState& bs, int B, int Rp, int K, int bos, const int32_t* len_src, int32_t* len_exp, hipStream_t st);
// z [Rp, V] = logits incl. bias.  Step j of max_len; K <= 16.  fast_exp: the hardware exponential in the rows'
// log-sum-exp (the 16-bit path).
void launch_beam_select(const float* z, int V, const BeamState& bs, int B, int K, int j, int max_len, int eos, float alpha,
                        hipStream_t st, int fast_exp = 0);
void launch_beam_reorder(int prec, const BeamReorder& ro, const BeamState& bs, int R, int H, int L, hipStream_t st);
void launch_beam_finish(const BeamState& bs, int B, int K, int max_len, int pad, int32_t* out_ids, int32_t* out_len, float* out_score,
                        hipStream_t st);

}  // namespace cmt
