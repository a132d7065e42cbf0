// Host side of the C ABI (include/cytonmt_hip.h): argument validation, the workspace layout, and
// the kernel schedules of a training step, of greedy decoding and of beam search.  No arithmetic of
// the method happens here.
//
// Schedule of one training step:
//   gathers -> encoder bottom layer (input GEMM batched over all source positions, then both
//   directions in one fused recurrent kernel per position) -> upper encoder layers as a wavefront
//   over (layer, position) -> attention-key hoist K = H_s W_a -> decoder time loop (per step: one
//   fused LSTM kernel per layer, attention, attentional tanh layer) -> output layer in slabs of
//   target positions (projection + log-sum-exp partials, e -> dz rescale, dH_o and dW_o GEMMs) ->
//   decoder loop backwards -> deferred attention gradients -> encoder loops backwards.  Everything
//   that does not feed a recurrence — transposes, weight gradients as GEMMs batched over all time
//   steps (the paper's calculateGradient accumulation becomes the k = B*T contraction), dW_o, the
//   deterministic embedding scatters — runs on the library's second stream and is joined before the
//   step ends on the caller's stream.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <functional>
#include <chrono>
#include <string>
#include <vector>

#include "../../include/cytonmt_hip.h"
#include "kernels.h"

using namespace cmt;

namespace {

struct ParamInfo { std::string name; int64_t rows, cols; size_t off; };

// one LSTM (layer, direction)
struct LD {
  int Kin = 0, Hh = 0;
  int ph = 0, pg = 0;                // row pitches (elements) of Hst and dG: Hh + 8, 4Hh + 8 (see ACT_PAD)
  size_t w_off = 0, b_off = 0;       // element offsets in the flat parameter vector
  char* W = nullptr;                 // T [4Hh, Kin+Hh]
  char* Wt = nullptr;                // T [Kin+Hh, 4Hh]
  char* Hst = nullptr;               // T [(Lmax+1), Bp, Hh]
  float* Cst = nullptr;              // [(Lmax+1), Bp, Hh]
  float* Gs = nullptr;               // [Lmax, Bp, 4Hh] gate activations
  float* Gx = nullptr;               // [Lmax, Bp, 4Hh] batched input pre-activations (may be null)
  char* dG = nullptr;                // T [Lmax, Bp, 4Hh]
  char* dGT = nullptr;               // T [4Hh, Lmax*Bp]
  char* HstT = nullptr;              // T [Hh, (Lmax+1)*Bp]
  char* Yd = nullptr;                // T [Lmax, Bp, Hh] the layer's output after dropout (row pitch ph) ...
  char* YdT = nullptr;               // ... and its transpose [Hh, L*Bp]; used only while dropout is on
  float* dh = nullptr; float* dc = nullptr;   // [Bp, Hh]
  float* bwdp = nullptr;             // [8][Bp][2Hh] backward step-GEMM planes
  // fragment-major copies read by the per-step kernels (bf16 path, Hh a multiple of 32; see fm_offset)
  int Kstep = 0;                     // width of the per-step input segment: the x columns [Kin - Kstep, Kin) of W
  char* Wfm = nullptr;               // gate rows of W, columns [Kin - Kstep, Kin + Hh)
  char* HstF = nullptr;              // [(Lmax+1)] slots of [Bp, Hh]
  char* YdF = nullptr;               // [Lmax] slots of [Bp, Hh] (the layer's output after dropout)
  bool fm = false;
  char* WtF = nullptr;               // W^T [Kin+Hh, 4Hh] (backward step GEMMs; needs Kin a multiple of 16)
  char* dGF = nullptr;               // [Lmax] slots of [Bp, 4Hh]
  bool fmb = false;
};

// Row pitch padding of the per-step activation operands.  The step kernels read 16 sentences x 64
// bytes per fragment load; with a power-of-two pitch those 16 segments fall on the same cache banks
// (measured: 14.3 -> 11.0 us for the decoder LSTM step with 16 bytes of padding; rows kept 128-byte aligned by
// padding with 64 elements instead: 11.6 us against 9.8 us, 32 / 72 / 136 elements: 10.0 - 10.2 us).
constexpr int ACT_PAD = 8;

// Row capacity of an output-layer slab: CE_SLAB_MAX_ROWS unless CMT_CE_SLAB_ROWS asks for less (a multiple of 256
// from 256 up; read whenever a handle or a size query is set up, so both see the same value).
static int ce_cap_env() {
  const char* e = getenv("CMT_CE_SLAB_ROWS");
  const int v = e ? atoi(e) / 256 * 256 : 0;
  return v >= 256 ? std::min(CE_SLAB_MAX_ROWS, v) : CE_SLAB_MAX_ROWS;
}

struct Bump {
  char* base; size_t off = 0;
  explicit Bump(char* b) : base(b) {}
  char* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    char* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

}  // namespace

struct cmt_handle {
  cmt_config cfg;
  int prec = 0; size_t esz = 4;
  hipStream_t st = nullptr;
  float* params = nullptr; float* grads = nullptr; char* ws = nullptr;
  size_t nparams = 0;
  std::vector<ParamInfo> table;
  std::string err;
  int Bpm = 0;                          // padded max batch
  int PH = 0;                           // row pitch of HoBuf, Cs, dPre: H + ACT_PAD
  // last-step shape
  int B = 0, Bp = 0, S = 0, T = 0;
  bool have_step = false;
  // pinned host
  float* h_loss = nullptr; int* h_flags = nullptr;

  // parameter working copies
  char* Pc = nullptr;                   // T copy of the flat parameter vector (bf16 path) or the master itself
  std::vector<LD> enc, dec;             // enc: [l0 fwd, l0 bwd, l1, ...]; dec: [l0, l1, ...]
  size_t off_Esrc = 0, off_Etgt = 0, off_Wa = 0, off_Wc = 0, off_Wo = 0, off_Bo = 0;
  char *WaT = nullptr, *WcT = nullptr, *WoT = nullptr;

  // source side
  char* Xs = nullptr; float* mask_s = nullptr; int32_t* tok_s = nullptr; int32_t* len_s = nullptr;
  char* Y0 = nullptr; char* Y0T = nullptr; char* Kmat = nullptr;
  float* Pmat = nullptr; char* PmatT = nullptr;   // the source states through the context half of W_c, [S * Bp, H] in fp32 and in
                                        // the operand type (Eq. 7 regrouped)
  int att_proj = 1;                     // attention on the projected source rows (see enqueue_step): 1 both decoder loops,
                                        // 2 the forward loop alone, 0 neither
  float* dHs = nullptr; char* dK = nullptr; char* dKT = nullptr;
  float* dYa = nullptr; float* dXs = nullptr; char* XsT = nullptr;
  // target side
  char* Xt = nullptr; float* mask_t = nullptr; int32_t* tok_t = nullptr; int32_t* labels = nullptr; int32_t* len_t = nullptr;
  char* HoBuf = nullptr; char* HoBufT = nullptr; char* Cs = nullptr; char* CsT = nullptr;
  float* att_a = nullptr; float* att_ds = nullptr; float* dCs = nullptr; float* dots = nullptr;
  float* att_s = nullptr;               // [Tmax, Bp, Smax] attention scores of every step of the last training step
  char* dPre = nullptr; char* dPreT = nullptr;
  float* dHoCE = nullptr;
  float* dHt = nullptr; float* wcp = nullptr;
  float* dXt = nullptr; char* XtT = nullptr;
  float *pmax = nullptr, *psum = nullptr, *zy = nullptr, *lse = nullptr, *nll = nullptr, *rowscale = nullptr;
  // the output layer works on the valid target positions only, numbered densely on the device
  int32_t *ce_pos = nullptr, *ce_row = nullptr, *ce_nvalid = nullptr, *labels_c = nullptr;
  char* Hoc = nullptr; char* HocT = nullptr;   // H_o (as the output layer sees it) of the valid positions, and its transpose
  float* loss = nullptr; int* flags = nullptr; float* colscr = nullptr;
  char* dzs = nullptr; char* dzTs = nullptr; float* dbo_parts = nullptr;
  std::vector<GemmProb> dw_group;       // weight-gradient GEMMs collected for one grouped launch (flush_dw_group)
  int ce_rows = 0, ce_pitch = 0;        // row capacity of an output-layer slab and the row pitch of its buffers
  int ce_cap = ce_cap_env();            // upper bound of ce_rows
  float* gsplit = nullptr; size_t gsplit_floats = 0;   // split-k planes of dH_o = dz W_o (also the probes' scratch)
  float* gsplit2 = nullptr; size_t gsplit2_floats = 0; // split-k planes of the second stream's GEMMs (fp32 path)
  hipStream_t side = nullptr;           // library-owned second stream for work off the recurrences' critical path
  std::vector<hipEvent_t> ev; size_t ev_next = 0;
  int use_side = 1;
  char* dzs2 = nullptr; char* dzTs2 = nullptr;
  char* WcF = nullptr; char* WcTF = nullptr;  // fragment-major W_c [H, 2H] and W_c^T [2H, H]
  char* WoF = nullptr;                        // fragment-major W_o [V, H] (greedy decoding's logits; V a multiple of 16)
  char* CsF = nullptr; char* dPreF = nullptr; // fragment-major copies of the contexts and of dpre, [Tmax] slots of [Bp, H]
  char* HoFeedF = nullptr;              // fragment-major copy of the H_o rows fed to the decoder's bottom layer, [(Tmax+1)] slots of [Bp, H]
  // decoding (greedy, beam): the bottom decoder layer contracts [embedding; H_o; h] in one step, so it needs the gate
  // rows of all E + 2H columns of its weights and its input [Bp, E + H] in fragment-major form
  char* Wdec0F = nullptr; char* xcatF = nullptr;
  int kb_bwd = 0, kb_wc = 0;            // caps on the k blocks of the backward step GEMMs (0 = default)
  int kb_bwd_dec = 0;                   // the same for the decoder's k-split form (one instance per launch)
  // Workgroup caps of the second stream's GEMMs (weight gradients; dW_o), 0 = none, -1 = by batch width: with all
  // 256 CUs taken by 256 x 256 tiles for tens of microseconds at a time, the recurrences' kernels on the caller's
  // stream queue behind them; capped at 128 workgroups the GEMMs take twice as long (still hidden) and leave half the
  // chip free.  Step time capped / uncapped, ms: medium 9.83 / 9.96, attn 11.03 / 11.12, small (fp32) 10.57 / 10.90;
  // at 128 sentences (large) 24.82 / 24.73, so the caps apply up to 64 sentences.  Env CMT_SIDE_WGS, CMT_SIDE_WGS_WO.
  int side_wgs = -1, side_wgs_wo = -1;
  int side_cap(int v) const { return v >= 0 ? v : (Bp <= 64 ? 128 : 0); }
  int wc_whole_k = 1;                   // fused decoder loop: dpre W_c with the whole k range per workgroup (env CMT_WC_WHOLE_K)
  // backward loops that use the whole-k step GEMM with the consumer in its epilogue (env CMT_BWD_FUSED, a bit
  // mask): 1 = decoder (up to 128 sentences: 8.1 against 8.7 ms for the large workload's backward loop; wider
  // batches keep the k-split GEMM + pointwise pair), 2 = upper encoder layers, 4 = bottom encoder layer.  Without
  // the switch (bwd_fused_auto) bits 1 and 4 are set and the upper encoder layers choose per step: their launches
  // carry up to L - 1 layer-steps, each re-reading all gate gradients from L2 in the fused form, so it wins while
  // (L - 1) * Bp * H^2 is small (step time fused / pair, ms: 512 x 2 layers 5.07 / 5.22, 512 x 4 6.89 / 7.09,
  // 1024 x 2 6.30 / 6.45, 512 x 2 at 32 sentences x 120 positions 11.77 / 12.13; 1024 x 4 at 64 sentences
  // 9.43 / 9.41; at 128 sentences 26.4 / 25.3): fused up to 2^27.
  int bwd_fused = 5;
  bool bwd_fused_auto = true;
  // phase timing of a step on the caller's stream (measurement aid, env CMT_PHASE_TIMING=1)
  int phase_timing = 0;
  std::vector<hipEvent_t> phase_ev; std::vector<const char*> phase_name; size_t phase_n = 0;
  std::vector<double> phase_host;       // host clock (ms) when each mark was enqueued
  // regularisation of the next steps (cmt_set_regularization)
  float drop_p = 0.f, drop_scale = 1.f, ls_eps = 0.f;
  unsigned drop_thresh = 0; unsigned long long drop_seed = 0;
  // greedy decoding
  char* xcat = nullptr; int ldxcat = 0; // decoder bottom-layer input [emb(y_{j-1}) ; H_o^{<j-1>}] of the current step
  int32_t* dec_tok = nullptr; int32_t* dec_done = nullptr; float* dec_mask = nullptr; float* logits = nullptr;
  // beam search: encoder outputs repeated per hypothesis row, and the search state
  char* Hs_exp = nullptr; char* K_exp = nullptr; int32_t* len_exp = nullptr;
  BeamState beam{};
  char* HoDrop = nullptr;               // H_o after dropout: what the output layer and the input feed read
  float* psz = nullptr;                 // per-group sums of logits (label smoothing)
  size_t ws_bytes = 0;

  const char* Pw(size_t off) const { return Pc + off * esz; }
};

namespace {

int round_up(int v, int m) { return (v + m - 1) / m * m; }

// jobs for launch_fill_multi / launch_copy2d_multi (units of 32-bit words; esz = bytes per T element)
void add_fill(std::vector<FillJob>& v, void* p, size_t elems, size_t esz) { v.push_back(FillJob{p, elems * esz / 4}); }
void add_copy(std::vector<CopyJob>& v, const void* s, int lds, void* d, int ldd, int rows, int cols, size_t esz) {
  const int f = (int)(4 / esz);                    // elements per word: row pitches and widths are multiples of it
  v.push_back(CopyJob{s, lds / f, d, ldd / f, rows, cols / f});
}

bool config_ok(const cmt_config* c, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (!c) return bad("null config");
  if (c->src_vocab < 8 || c->tgt_vocab < 8 || c->src_vocab % 8 || c->tgt_vocab % 8) return bad("vocabulary sizes must be positive multiples of 8");
  if (c->emb_dim < 8 || c->emb_dim % 8 || c->emb_dim > 2048) return bad("emb_dim must be a multiple of 8 in [8, 2048]");
  if (c->hidden < 16 || c->hidden % 16 || c->hidden > 1024) return bad("hidden must be a multiple of 16 in [16, 1024]");
  if (c->layers < 1 || c->layers > 8) return bad("layers must be in [1, 8]");
  if (c->max_batch < 1 || c->max_batch > 4096) return bad("max_batch must be in [1, 4096]");
  if (c->max_src_len < 1 || c->max_src_len > 512) return bad("max_src_len must be in [1, 512]");
  if (c->max_tgt_len < 1 || c->max_tgt_len > 4096) return bad("max_tgt_len must be in [1, 4096]");
  if (c->precision != 0 && c->precision != 1) return bad("precision must be 0 (fp32) or 1 (bf16)");
  if (c->bos_id < 0 || c->bos_id >= c->tgt_vocab) return bad("bos_id outside the target vocabulary");
  if (c->pad_id < 0 || c->pad_id >= c->tgt_vocab || c->pad_id >= c->src_vocab) return bad("pad_id outside a vocabulary");
  return true;
}

void build_table(const cmt_config& c, std::vector<ParamInfo>& t, size_t& total) {
  const int64_t Vs = c.src_vocab, Vt = c.tgt_vocab, E = c.emb_dim, H = c.hidden, Hd = H / 2;
  size_t off = 0;
  auto add = [&](const std::string& n, int64_t r, int64_t cc) { t.push_back({n, r, cc, off}); off += (size_t)(r * cc); };
  add("E_src", Vs, E); add("E_tgt", Vt, E);
  add("enc.l0.fwd.W", 4 * Hd, E + Hd); add("enc.l0.fwd.b", 4 * Hd, 1);
  add("enc.l0.bwd.W", 4 * Hd, E + Hd); add("enc.l0.bwd.b", 4 * Hd, 1);
  for (int l = 1; l < c.layers; ++l) {
    add("enc.l" + std::to_string(l) + ".W", 4 * H, 2 * H); add("enc.l" + std::to_string(l) + ".b", 4 * H, 1);
  }
  add("dec.l0.W", 4 * H, E + 2 * H); add("dec.l0.b", 4 * H, 1);
  for (int l = 1; l < c.layers; ++l) {
    add("dec.l" + std::to_string(l) + ".W", 4 * H, 2 * H); add("dec.l" + std::to_string(l) + ".b", 4 * H, 1);
  }
  add("W_a", H, H); add("W_c", H, 2 * H); add("W_o", Vt, H); add("B_o", Vt, 1);
  total = off;
}

size_t find_off(const std::vector<ParamInfo>& t, const std::string& n) {
  for (auto& p : t) if (p.name == n) return p.off;
  return 0;
}

// Carves the workspace.  With base == nullptr only the size is computed.
size_t layout(cmt_handle* h, char* base) {
  const cmt_config& c = h->cfg;
  const size_t esz = h->esz;
  const int E = c.emb_dim, H = c.hidden, Hd = H / 2, L = c.layers;
  const int Bp = h->Bpm, Sm = c.max_src_len, Tm = c.max_tgt_len;
  const size_t Ms = (size_t)Sm * Bp, Mt = (size_t)Tm * Bp;
  Bump a(base);
  h->PH = H + ACT_PAD;
  const size_t PH = h->PH;
  h->Pc = c.precision ? a.take(h->nparams * esz) : (char*)h->params;
  auto ld_alloc = [&](LD& d, int Kin, int Hh, int Lm, bool gx, int Kstep) {
    d.Kin = Kin; d.Hh = Hh; d.ph = Hh + ACT_PAD; d.pg = 4 * Hh + ACT_PAD;
    const size_t M = (size_t)Lm * Bp;
    d.Kstep = Kstep;
    d.fm = c.precision && Hh % 32 == 0 && Kstep % 32 == 0;
    if (d.fm) {
      d.Wfm = a.take((size_t)4 * Hh * (Kstep + Hh) * esz);
      d.HstF = a.take((M + Bp) * Hh * esz);
      d.YdF = a.take(M * Hh * esz);
    }
    d.fmb = c.precision && Hh % 32 == 0 && Kin % 16 == 0;
    if (d.fmb) {
      d.WtF = a.take((size_t)(Kin + Hh) * 4 * Hh * esz);
      d.dGF = a.take(M * 4 * Hh * esz);
    }
    d.Wt = a.take((size_t)(Kin + Hh) * 4 * Hh * esz);
    d.Hst = a.take((M + Bp) * d.ph * esz);
    d.Cst = (float*)a.take((M + Bp) * Hh * 4);
    d.Gs = (float*)a.take(M * 4 * Hh * 4);
    d.Gx = gx ? (float*)a.take(M * 4 * Hh * 4) : nullptr;
    d.dG = a.take(M * d.pg * esz);
    d.dGT = a.take(M * 4 * Hh * esz);
    d.HstT = a.take((M + Bp) * Hh * esz);
    d.dh = (float*)a.take((size_t)Bp * Hh * 4);
    d.dc = (float*)a.take((size_t)Bp * Hh * 4);
    d.bwdp = (float*)a.take((size_t)8 * Bp * 2 * Hh * 4);
    d.Yd = a.take(M * d.ph * esz);                 // the layer's output after dropout, and its transpose
    d.YdT = a.take(M * Hh * esz);
  };
  h->enc.assign(L + 1, LD());
  h->dec.assign(L, LD());
  // per-step input segment: none for the layers whose input part is batched over time (bottom encoder layers,
  // encoder layer 1), the fed H_o for the decoder's bottom layer, the layer below's state for the others
  ld_alloc(h->enc[0], E, Hd, Sm, true, 0);
  ld_alloc(h->enc[1], E, Hd, Sm, true, 0);
  for (int l = 1; l < L; ++l) ld_alloc(h->enc[l + 1], H, H, Sm, true, l == 1 ? 0 : H);
  ld_alloc(h->dec[0], E + H, H, Tm, true, H);
  for (int l = 1; l < L; ++l) ld_alloc(h->dec[l], H, H, Tm, false, H);
  if (c.precision && H % 32 == 0) {
    h->HoFeedF = a.take((Mt + Bp) * H * esz);
    h->WcF = a.take((size_t)2 * H * H * esz); h->WcTF = a.take((size_t)2 * H * H * esz);
    h->CsF = a.take(Mt * H * esz); h->dPreF = a.take(Mt * H * esz);
    if (c.tgt_vocab % 16 == 0) h->WoF = a.take((size_t)c.tgt_vocab * H * esz);
    if (E % 32 == 0) { h->Wdec0F = a.take((size_t)4 * H * (E + 2 * H) * esz); h->xcatF = a.take((size_t)Bp * (E + H) * esz); }
  }
  h->WaT = a.take((size_t)H * H * esz);
  h->WcT = a.take((size_t)2 * H * H * esz);
  h->WoT = a.take((size_t)H * c.tgt_vocab * esz);
  // source side
  h->Xs = a.take(Ms * E * esz); h->XsT = a.take(Ms * E * esz);
  h->mask_s = (float*)a.take(Ms * 4); h->tok_s = (int32_t*)a.take(Ms * 4); h->len_s = (int32_t*)a.take((size_t)Bp * 4);
  h->Y0 = a.take(Ms * H * esz); h->Y0T = a.take(Ms * H * esz); h->Kmat = a.take(Ms * H * esz);
  h->Pmat = (float*)a.take(Ms * H * 4); h->PmatT = a.take(Ms * H * esz);
  h->dHs = (float*)a.take(Ms * H * 4); h->dK = a.take(Ms * H * esz); h->dKT = a.take(Ms * H * esz);
  h->dYa = (float*)a.take(Ms * H * 4);
  h->dXs = (float*)a.take(Ms * E * 4);
  // target side
  h->Xt = a.take(Mt * E * esz); h->XtT = a.take(Mt * E * esz);
  h->mask_t = (float*)a.take(Mt * 4); h->tok_t = (int32_t*)a.take(Mt * 4); h->labels = (int32_t*)a.take(Mt * 4);
  h->len_t = (int32_t*)a.take((size_t)Bp * 4);
  h->HoBuf = a.take((Mt + Bp) * PH * esz); h->HoBufT = a.take((Mt + Bp) * H * esz);
  h->HoDrop = a.take((Mt + Bp) * PH * esz);
  h->ldxcat = E + H + ACT_PAD;
  h->xcat = a.take((size_t)Bp * h->ldxcat * esz);
  h->dec_tok = (int32_t*)a.take((size_t)Bp * 4); h->dec_done = (int32_t*)a.take((size_t)Bp * 4);
  h->dec_mask = (float*)a.take((size_t)Bp * 4);
  h->logits = (float*)a.take((size_t)Bp * c.tgt_vocab * 4);
  h->Hs_exp = a.take(Ms * H * esz); h->K_exp = a.take(Ms * H * esz);
  h->len_exp = (int32_t*)a.take((size_t)Bp * 4);
  {
    BeamState& bs = h->beam;
    bs.cum = (float*)a.take((size_t)Bp * 4); bs.new_cum = (float*)a.take((size_t)Bp * 4); bs.mask = (float*)a.take((size_t)Bp * 4);
    bs.tok = (int32_t*)a.take((size_t)Bp * 4); bs.new_tok = (int32_t*)a.take((size_t)Bp * 4);
    bs.parent = (int32_t*)a.take((size_t)Bp * 4); bs.nlive = (int32_t*)a.take((size_t)Bp * 4);
    bs.fin_score = (float*)a.take((size_t)Bp * 4); bs.fin_step = (int32_t*)a.take((size_t)Bp * 4);
    bs.fin_par = (int32_t*)a.take((size_t)Bp * 4); bs.fin_tok = (int32_t*)a.take((size_t)Bp * 4);
    bs.hist_tok = (int32_t*)a.take(Mt * 4); bs.hist_par = (int32_t*)a.take(Mt * 4);
    bs.hist_ld = Bp;
    bs.row_lse = (float*)a.take((size_t)Bp * 4);
    bs.cand_z = (float*)a.take((size_t)Bp * 16 * 4); bs.cand_tok = (int32_t*)a.take((size_t)Bp * 16 * 4);
  }
  h->Cs = a.take(Mt * PH * esz); h->CsT = a.take(Mt * H * esz);
  h->att_a = (float*)a.take(Mt * Sm * 4); h->att_ds = (float*)a.take(Mt * Sm * 4);
  h->dCs = (float*)a.take(Mt * H * 4);
  h->dots = (float*)a.take((size_t)Bp * Sm * 4);
  h->att_s = (float*)a.take(Mt * Sm * 4);
  h->dPre = a.take(Mt * PH * esz); h->dPreT = a.take(Mt * H * esz);
  h->dHoCE = (float*)a.take(Mt * H * 4);
  h->dHt = (float*)a.take((size_t)Bp * H * 4);
  h->wcp = (float*)a.take((size_t)8 * Bp * 2 * H * 4);
  h->dXt = (float*)a.take(Mt * E * 4);
  const int np = ce_num_partials(c.tgt_vocab);
  // output-layer slabs: one slab for the whole batch up to the cap, else full slabs of the cap and a remainder
  h->ce_rows = (int)std::min<size_t>((size_t)h->ce_cap, (Mt + 255) / 256 * 256);
  h->ce_pitch = ce_slab_pitch(h->ce_rows);
  const size_t ce_slabs = (Mt + h->ce_rows - 1) / h->ce_rows;
  const size_t slab_elems = (size_t)h->ce_pitch * c.tgt_vocab;      // elements of a slab buffer (e / dz, and dz^T)
  {   // per slab a [np, pitch] block of partials (slab sl starts at sl * np * pitch)
    const size_t bytes = ce_slabs * h->ce_pitch * np * 4;
    h->pmax = (float*)a.take(bytes); h->psum = (float*)a.take(bytes); h->psz = (float*)a.take(bytes);
  }
  h->zy = (float*)a.take(Mt * 4); h->lse = (float*)a.take(Mt * 4); h->nll = (float*)a.take(Mt * 4);
  h->rowscale = (float*)a.take(Mt * 4);
  h->ce_pos = (int32_t*)a.take(Mt * 4); h->ce_row = (int32_t*)a.take(Mt * 4); h->labels_c = (int32_t*)a.take(Mt * 4);
  h->ce_nvalid = (int32_t*)a.take(256);
  h->Hoc = a.take(Mt * PH * esz); h->HocT = a.take(Mt * H * esz);
  h->loss = (float*)a.take(256); h->flags = (int*)a.take(256);
  h->colscr = (float*)a.take((size_t)16 * 4 * H * 4);
  h->dzs = a.take(slab_elems * esz); h->dzTs = a.take(slab_elems * esz);
  h->dbo_parts = (float*)a.take((Mt / 64 + Mt / 256 + 4) * c.tgt_vocab * 4);
  {   // split-k planes of dH_o = dz W_o of a slab (k = the vocabulary): 16 planes, at most 256 MB, at least 1 MB
    const size_t slab_rows = std::min<size_t>(Mt, (size_t)h->ce_rows);
    h->gsplit_floats = std::max((size_t)1 << 18, std::min((size_t)64 << 20, 16 * slab_rows * H));
  }
  h->gsplit = (float*)a.take(h->gsplit_floats * 4);
  h->gsplit2_floats = c.precision ? 0 : std::min((size_t)8 << 20, (size_t)16 * 4 * H * std::max(E, H));
  h->gsplit2 = (float*)a.take(h->gsplit2_floats * 4);
  if (ce_slabs > 1) {                             // a second pair, so that slab s + 1 starts while dW_o of slab s still runs
    h->dzs2 = a.take(slab_elems * esz); h->dzTs2 = a.take(slab_elems * esz);
  } else {
    h->dzs2 = h->dzs; h->dzTs2 = h->dzTs;
  }
  return (a.off + 255) & ~(size_t)255;
}

void bind_params(cmt_handle* h) {
  const cmt_config& c = h->cfg;
  auto& t = h->table;
  h->off_Esrc = find_off(t, "E_src"); h->off_Etgt = find_off(t, "E_tgt");
  h->off_Wa = find_off(t, "W_a"); h->off_Wc = find_off(t, "W_c");
  h->off_Wo = find_off(t, "W_o"); h->off_Bo = find_off(t, "B_o");
  auto bind = [&](LD& d, const std::string& n) {
    d.w_off = find_off(t, n + ".W"); d.b_off = find_off(t, n + ".b");
    d.W = h->Pc + d.w_off * h->esz;
  };
  bind(h->enc[0], "enc.l0.fwd"); bind(h->enc[1], "enc.l0.bwd");
  for (int l = 1; l < c.layers; ++l) bind(h->enc[l + 1], "enc.l" + std::to_string(l));
  for (int l = 0; l < c.layers; ++l) bind(h->dec[l], "dec.l" + std::to_string(l));
}

// refresh the kernels' working copies of the parameters: operand-type cast, transposes
void refresh_params(cmt_handle* h, bool cast = true) {
  const cmt_config& c = h->cfg;
  const int H = c.hidden, p = h->prec;
  hipStream_t st = h->st;
  if (p && cast) launch_cast(1, h->params, h->Pc, h->nparams, st);
  auto tr = [&](LD& d) {
    launch_transpose(p, d.W, d.Kin + d.Hh, d.Wt, 4 * d.Hh, 4 * d.Hh, d.Kin + d.Hh, st);
    if (d.fm) launch_fm_pack_lstm_weights(d.W, d.Kin + d.Hh, d.Kin - d.Kstep, d.Kstep + d.Hh, d.Hh, d.Wfm, st);
    if (d.fmb) launch_fm_pack(d.Wt, 4 * d.Hh, d.Kin + d.Hh, 4 * d.Hh, d.WtF, st);
  };
  for (auto& d : h->enc) tr(d);
  for (auto& d : h->dec) tr(d);
  launch_transpose(p, h->Pw(h->off_Wa), H, h->WaT, H, H, H, st);
  launch_transpose(p, h->Pw(h->off_Wc), 2 * H, h->WcT, H, H, 2 * H, st);
  if (h->WcF) {
    launch_fm_pack(h->Pw(h->off_Wc), 2 * H, H, 2 * H, h->WcF, st);
    launch_fm_pack(h->WcT, H, 2 * H, H, h->WcTF, st);
    if (h->WoF) launch_fm_pack(h->Pw(h->off_Wo), H, c.tgt_vocab, H, h->WoF, st);
    if (h->Wdec0F) launch_fm_pack_lstm_weights(h->dec[0].W, c.emb_dim + 2 * H, 0, c.emb_dim + 2 * H, H, h->Wdec0F, st);
  }
  launch_transpose(p, h->Pw(h->off_Wo), H, h->WoT, c.tgt_vocab, c.tgt_vocab, H, st);
}

int fail(cmt_handle* h, int code, const std::string& msg) {
  if (h) h->err = msg;
  return code;
}
int hip_fail(cmt_handle* h, hipError_t e, const char* what) {
  return fail(h, CMT_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

// ------------------------------------------------------------------------------------------------
// the schedule
// ------------------------------------------------------------------------------------------------
// make stream `to` wait for everything enqueued so far on stream `from`
void stream_after(cmt_handle* h, hipStream_t to, hipStream_t from) {
  if (to == from) return;
  hipEvent_t e = h->ev[h->ev_next++ % h->ev.size()];
  (void)hipEventRecord(e, from);
  (void)hipStreamWaitEvent(to, e, 0);
}

void weight_grads(cmt_handle* h, LD& d, int Lsteps, const std::vector<std::pair<const char*, int>>& segs /* (XT ptr, ld) */,
                  const std::vector<int>& seg_k, hipStream_t st) {
  // dW[:, segment] = dG^T * X_segment as one GEMM with k = Lsteps * Bp; db = column sums of dG
  const int p = h->prec, Bp = h->Bp, Hh = d.Hh;
  const int M = Lsteps * Bp;
  launch_transpose(p, d.dG, d.pg, d.dGT, M, M, 4 * Hh, st);
  float* dW = h->grads + d.w_off;
  int col = 0;
  for (size_t i = 0; i < segs.size(); ++i) {
    h->dw_group.push_back(GemmProb{d.dGT, segs[i].first, dW + col, M, segs[i].second, d.Kin + Hh, 4 * Hh, seg_k[i], M, 0});
    col += seg_k[i];
  }
  launch_colsum(p, d.dG, d.pg, M, 4 * Hh, h->colscr, h->grads + d.b_off, st);
}
// launches what weight_grads (and the callers that add W_c / W_a problems) have collected, as one queue of tiles
void flush_dw_group(cmt_handle* h, hipStream_t st) {
  launch_gemm_nt_group(h->prec, h->dw_group.data(), (int)h->dw_group.size(), st, h->gsplit2, h->gsplit2_floats,
                       st != h->st ? h->side_cap(h->side_wgs) : 0);
  h->dw_group.clear();
}

// marks the start of a phase of the step on the caller's stream (only when phase timing is on)
void phase_mark(cmt_handle* h, const char* name) {
  if (!h->phase_timing) return;
  if (h->phase_n >= h->phase_ev.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    h->phase_ev.push_back(e); h->phase_name.push_back(name);
  }
  h->phase_name[h->phase_n] = name;
  if (h->phase_host.size() <= h->phase_n) h->phase_host.resize(h->phase_n + 1);
  h->phase_host[h->phase_n] = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
  (void)hipEventRecord(h->phase_ev[h->phase_n++], h->st);
}

// The output layer's slabs: full slabs of the handle's slab capacity and one remainder (a single slab whenever
// the batch fits).  Returns the rows of all slabs but the last.
int ce_slab_plan(const cmt_handle* h, int Mt, int* nslab_out) {
  *nslab_out = (Mt + h->ce_rows - 1) / h->ce_rows;
  return h->ce_rows;
}

// dropout sites (the oracle and the tests use the same numbering): encoder layer l output, decoder
// layer l output, H_o
constexpr int DROP_SITE_ENC = 0, DROP_SITE_DEC = 16, DROP_SITE_HO = 32;
DropSpec drop_spec(const cmt_handle* h, int site, int t) {
  DropSpec d;
  if (h->drop_p > 0.f) {
    const unsigned long long H = (unsigned long long)h->cfg.hidden;
    d.on = 1; d.thresh = h->drop_thresh; d.scale = h->drop_scale; d.width = h->cfg.hidden;
    d.key0 = h->drop_seed + ((unsigned long long)site << 48) + (unsigned long long)t * (unsigned long long)h->B * H;
  }
  return d;
}

// the cell backward of decoder layer l at step j; dy / dhrec are filled in by the caller
LstmBwdPoint dec_cell(cmt_handle* h, int l, int j) {
  const int H = h->cfg.hidden, Bp = h->Bp;
  const size_t BH = (size_t)Bp * H;
  LD& e = h->dec[l];
  LstmBwdPoint q;
  q.dy = Planes{nullptr, 0, 0, 0}; q.dy_col = 0; q.dhrec = Planes{nullptr, 0, 0, 0}; q.dhrec_col = 0;
  q.dh = e.dh; q.dc = e.dc;
  q.gsave = e.Gs + (size_t)j * Bp * 4 * H;
  q.cprev = e.Cst + j * BH; q.cnext = e.Cst + (j + 1) * BH;
  q.mask = h->mask_t + (size_t)j * Bp;
  q.dg = e.dG + (size_t)j * Bp * e.pg * h->esz; q.lddg = e.pg;
  if (e.fmb) q.dg_fm = e.dGF + (size_t)j * Bp * 4 * H * h->esz;
  return q;
}

// Backward step GEMM of decoder layer l at step j in its fused form: [dx; dh_prev] = dgates [W_x; W_h] with the
// whole contraction inside the workgroup.  The dx half feeds the cell backward of the layer below in the
// epilogue (bottom layer: the tanh backward of the previous step's H_o, which received it through the input
// feed); the dh_prev half is stored (one fp32 matrix per layer, the first Bp * H floats of bwdp) for that
// layer's next step.
StepBwd dec_bwd_gemm(cmt_handle* h, int l, int j) {
  const cmt_config& c = h->cfg;
  const int E = c.emb_dim, H = c.hidden, Bp = h->Bp, PH = h->PH;
  const size_t esz = h->esz, BP = (size_t)Bp * PH;
  const bool last = j == h->T - 1;
  LD& e = h->dec[l];
  StepBwd g{};
  g.dg = e.dG + (size_t)j * Bp * e.pg * esz; g.lddg = e.pg; g.K = 4 * H; g.ldw = 4 * H;
  BwdEpi store{};
  store.kind = BWD_EPI_STORE; store.ncols = H; store.hh = H; store.out = e.bwdp; store.ldout = H;
  if (l > 0) {
    g.Wt = e.Wt;
    BwdEpi& c0 = g.part[0];
    c0.kind = BWD_EPI_CELL_DY; c0.ncols = H; c0.hh = H;
    c0.cell = dec_cell(h, l - 1, j);
    c0.cell.drop_dy = drop_spec(h, DROP_SITE_DEC + l - 1, j);
    c0.cell.dhrec = Planes{h->dec[l - 1].bwdp, H, last ? 0 : 1, 0};
    g.part[1] = store;
  } else if (j > 0) {
    g.Wt = e.Wt + (size_t)E * 4 * H * esz;                       // rows [feed; h] of the bottom layer's W^T
    BwdEpi& t0 = g.part[0];
    t0.kind = BWD_EPI_TANH; t0.ncols = H; t0.hh = H;
    t0.dce = h->dHoCE; t0.pos = h->ce_pos + (size_t)(j - 1) * Bp; t0.Ho = h->HoBuf + j * BP * esz; t0.ldho = PH;
    t0.dpre = h->dPre + (j - 1) * BP * esz; t0.ldp = PH; t0.drop = drop_spec(h, DROP_SITE_HO, j - 1);
    if (h->dPreF) t0.dpre_fm = h->dPreF + (size_t)(j - 1) * Bp * H * esz;
    g.part[1] = store;
  } else {
    g.Wt = e.Wt + (size_t)(E + H) * 4 * H * esz;                 // H_o^{<-1>} is a constant: only dh_prev
    g.part[0] = store;
  }
  if (e.fmb) {                                                   // the same operands in fragment-major form
    g.dg_fm = e.dGF + (size_t)j * Bp * 4 * H * esz; g.Wt_fm = e.WtF;
    g.wt_tile0 = (l > 0 ? 0 : j > 0 ? E : E + H) / 16;
  }
  return g;
}

// forward step j of decoder layer l (layer 0 takes [H_o^{<j-1>}; h] per step, its embedding part is pre-batched)
void dec_lstm_fwd(cmt_handle* h, int l, int j) {
  const cmt_config& c = h->cfg;
  const int E = c.emb_dim, H = c.hidden, Bp = h->Bp;
  const size_t esz = h->esz, BH = (size_t)Bp * H, BP = (size_t)Bp * h->PH;
  LD& e = h->dec[l];
  LstmFwdDir d;
  const bool drop = h->drop_p > 0.f;
  if (l == 0) {
    d.x = (drop ? h->HoDrop : h->HoBuf) + j * BP * esz; d.ldx = h->PH; d.Kx = H; d.wx_off = E; d.wh_off = E + H;
    d.gx = e.Gx + (size_t)j * Bp * 4 * H; d.ldgx = 4 * H; d.bias = nullptr; d.ldw = E + 2 * H;
  } else {
    d.x = drop ? h->dec[l - 1].Yd + j * BP * esz : h->dec[l - 1].Hst + (j + 1) * BP * esz;
    d.ldx = e.ph; d.Kx = H; d.wx_off = 0; d.wh_off = H;
    d.gx = nullptr; d.ldgx = 0; d.bias = h->params + e.b_off; d.ldw = 2 * H;
  }
  d.hprev = e.Hst + j * BP * esz; d.ldh = e.ph; d.W = e.W;
  d.cprev = e.Cst + j * BH; d.mask = h->mask_t + (size_t)j * Bp;
  d.hnext = e.Hst + (j + 1) * BP * esz; d.ldhn = e.ph; d.cnext = e.Cst + (j + 1) * BH;
  d.gsave = e.Gs + (size_t)j * Bp * 4 * H; d.ycat = nullptr; d.ldy = 0;
  if (drop && l + 1 < c.layers) {                  // what the layer above reads
    d.ycat = e.Yd + j * BP * esz; d.ldy = e.ph; d.drop = drop_spec(h, DROP_SITE_DEC + l, j); d.drop_col0 = 0;
  }
  if (e.fm) {                                      // the contraction's operands in fragment-major form
    d.W_fm = e.Wfm;
    d.x_fm = l == 0 ? h->HoFeedF + j * BH * esz
                    : (drop ? h->dec[l - 1].YdF + j * BH * esz : h->dec[l - 1].HstF + (j + 1) * BH * esz);
    d.hprev_fm = e.HstF + j * BH * esz; d.hnext_fm = e.HstF + (j + 1) * BH * esz;
    if (d.ycat) d.ycat_fm = e.YdF + j * BH * esz;
  }
  launch_lstm_fwd(h->prec, &d, 1, Bp, H, h->st);
}

// Encoder forward for the batch whose source embeddings, masks and lengths are in the workspace
// (gather done by the caller): bottom layer (both directions per launch), upper layers as a
// wavefront, attention keys, and the decoder's initial states.  Returns H_s (top-layer states) and
// its row pitch.
// Attention and attentional layer of decoder step j on the projected source rows P_i = W_c1 H_s^i (Eq. 3-7
// regrouped: W_c [C_s; H_t] = sum_i a_i P_i + W_c2 H_t), two dependent launches: the scores together with the sums
// W_c2 H_t (both wait for the top layer's state alone), then softmax, mix, tanh -> H_o and its copies.
void dec_att_fwd_proj(cmt_handle* h, int j, int S, float* scores) {
  const int p = h->prec, H = h->cfg.hidden, L = h->cfg.layers, Bp = h->Bp, PH = h->PH;
  const size_t esz = h->esz, BH = (size_t)Bp * H, BP = (size_t)Bp * PH;
  const char* Ht = h->dec[L - 1].Hst + (j + 1) * BP * esz;
  StepGemm g{};
  g.a0 = nullptr; g.lda0 = PH; g.K0 = H; g.w0_off = 0; g.skip0 = 1;
  g.a1 = Ht; g.lda1 = PH; g.K1 = H; g.w1_off = H;
  g.W = h->Pw(h->off_Wc); g.ldw = 2 * H; g.N = H; g.mode = 3;
  g.out = h->wcp; g.ldout = H; g.plane_stride = BH;
  if (h->HoFeedF) { g.W_fm = h->WcF; g.a1_fm = h->dec[L - 1].HstF + (j + 1) * BH * esz; g.a0_fm = g.a1_fm; }
  AttOut o{};
  o.outT = h->HoBuf + (j + 1) * BP * esz; o.ldo = PH;
  if (h->drop_p > 0.f) { o.outD = h->HoDrop + (j + 1) * BP * esz; o.ldod = PH; o.drop = drop_spec(h, DROP_SITE_HO, j); }
  if (h->HoFeedF) o.outF = h->HoFeedF + (j + 1) * BH * esz;
  launch_att_fwd_proj(p, h->Kmat, H, h->PmatT, H, Ht, PH, g, o, h->len_s, S, Bp, H, scores, h->att_a + (size_t)j * Bp * S, h->st);
}
// The backward of the same on the projected rows, two dependent launches: the score gradients da_i = dC_s . H_s^i
// are dpre . P_i (fp32 rows), so they need dpre alone and ride in the launch of [dC_s ; dH_t] = dpre W_c, whose halves
// go where their readers want them (dC_s to its slot for the deferred gradients, the dH_t half beside it); then
// the softmax Jacobian, the gradient sent to the top layer's output and that layer's cell backward.
void dec_att_bwd_proj(cmt_handle* h, int j, int S, bool last) {
  const int p = h->prec, H = h->cfg.hidden, L = h->cfg.layers, Bp = h->Bp, PH = h->PH;
  const size_t esz = h->esz, BH = (size_t)Bp * H, BP = (size_t)Bp * PH;
  char* dpre = h->dPre + j * BP * esz;
  char* dpreF = h->dPreF ? h->dPreF + j * BH * esz : nullptr;
  StepBwd g{};
  g.dg = dpre; g.lddg = PH; g.K = H; g.Wt = h->WcT; g.ldw = H;
  g.part[0].kind = BWD_EPI_STORE; g.part[0].ncols = H; g.part[0].out = h->dCs + j * BH; g.part[0].ldout = H;
  g.part[1].kind = BWD_EPI_STORE; g.part[1].ncols = H; g.part[1].out = h->wcp; g.part[1].ldout = H;
  g.dg_fm = dpreF; g.Wt_fm = dpreF ? h->WcTF : nullptr; g.wt_tile0 = 0;
  const AttScores sc{h->Pmat, H, dpre, PH, h->len_s, S, H, h->dots, 1};
  launch_step_bwd_fused(p, &g, 1, Bp, h->st, &sc);
  LstmBwdPoint top = dec_cell(h, L - 1, j);
  top.dhrec = Planes{h->dec[L - 1].bwdp, H, last ? 0 : 1, 0};
  launch_att_bwd_mix(p, h->Kmat, H, Planes{h->wcp, H, 1, 0}, 0, h->att_a + (size_t)j * Bp * S, h->len_s, S, Bp, H, h->dots,
                     h->att_ds + (size_t)j * Bp * S, h->dHt, h->st, &top);
}

void enqueue_encoder(cmt_handle* h, int S, const char** Hs_out, int* ldHs_out) {
  const cmt_config& c = h->cfg;
  const int p = h->prec, E = c.emb_dim, H = c.hidden, Hd = H / 2, L = c.layers, Bp = h->Bp;
  const size_t esz = h->esz;
  hipStream_t st = h->st;
  const int Ms = S * Bp;
  const size_t BH = (size_t)Bp * H;
  const int PH = h->PH;
  const bool drop = h->drop_p > 0.f;
  const size_t BP = (size_t)Bp * PH;
  float* P = h->params;
  // ---- encoder layer 0: two directions ------------------------------------------------------------
  LD& ef = h->enc[0]; LD& eb = h->enc[1];
  for (LD* d : {&ef, &eb})
    launch_gemm_nt(p, h->Xs, E, d->W, E + Hd, Ms, 4 * Hd, E, d->Gx, nullptr, 4 * Hd, P + d->b_off, 0, st);
  const size_t BHd = (size_t)Bp * Hd, BPd = (size_t)Bp * ef.ph;
  {   // initial states of every encoder LSTM: zero, in one launch
    std::vector<FillJob> z;
    add_fill(z, ef.Hst, BPd, esz); add_fill(z, ef.Cst, BHd, 4);
    add_fill(z, eb.Hst + (size_t)S * BPd * esz, BPd, esz); add_fill(z, eb.Cst + (size_t)S * BHd, BHd, 4);
    if (ef.fm) { add_fill(z, ef.HstF, BHd, esz); add_fill(z, eb.HstF + (size_t)S * BHd * esz, BHd, esz); }
    for (int l = 1; l < L; ++l) {
      add_fill(z, h->enc[l + 1].Hst, BP, esz); add_fill(z, h->enc[l + 1].Cst, BH, 4);
      if (h->enc[l + 1].fm) add_fill(z, h->enc[l + 1].HstF, BH, esz);
    }
    launch_fill_multi(z.data(), (int)z.size(), st);
  }
  for (int k = 0; k < S; ++k) {
    const int tf = k, tb = S - 1 - k;
    LstmFwdDir d[2];
    for (int i = 0; i < 2; ++i) {
      LD& e = i ? eb : ef;
      const int t = i ? tb : tf;
      const int sp = i ? t + 1 : t, sn = i ? t : t + 1;
      d[i].x = nullptr; d[i].ldx = 0; d[i].Kx = 0;
      d[i].hprev = e.Hst + sp * BPd * esz; d[i].ldh = e.ph;
      d[i].W = e.W; d[i].ldw = E + Hd; d[i].wx_off = 0; d[i].wh_off = E;
      d[i].gx = e.Gx + (size_t)t * Bp * 4 * Hd; d[i].ldgx = 4 * Hd; d[i].bias = nullptr;
      d[i].cprev = e.Cst + sp * BHd; d[i].mask = h->mask_s + (size_t)t * Bp;
      d[i].hnext = e.Hst + sn * BPd * esz; d[i].ldhn = e.ph; d[i].cnext = e.Cst + sn * BHd;
      d[i].gsave = e.Gs + (size_t)t * Bp * 4 * Hd;
      d[i].ycat = h->Y0 + ((size_t)t * BH + (i ? Hd : 0)) * esz; d[i].ldy = H;
      if (L > 1) { d[i].drop = drop_spec(h, DROP_SITE_ENC + 0, t); d[i].drop_col0 = i ? Hd : 0; }
      if (e.fm) {
        d[i].W_fm = e.Wfm; d[i].hprev_fm = e.HstF + sp * BHd * esz; d[i].hnext_fm = e.HstF + sn * BHd * esz;
      }
    }
    launch_lstm_fwd(p, d, 2, Bp, Hd, st);
  }
  phase_mark(h, "encoder upper layers");
  // ---- encoder layers >= 1: a wavefront over (layer, position) ------------------------------------
  // Layer l at position t needs layer l-1 at t and itself at t-1, so all layers advance together
  // along diagonals: one launch carries up to L-1 layer-steps (S + L - 2 launches instead of
  // (L-1) S).  Layer 1 keeps its input part batched over all positions (the bottom layer is
  // complete by then); layers above take [x; h] W^T per step.
  const char* Yprev = h->Y0;                       // [S*Bp, H]
  int ldY = H;
  if (L > 1) {
    LD& e1 = h->enc[2];
    launch_gemm_nt(p, h->Y0, H, e1.W, 2 * H, Ms, 4 * H, H, e1.Gx, nullptr, 4 * H, P + e1.b_off, 0, st);
    for (int dg = 0; dg < S + L - 2; ++dg) {
      LstmFwdDir dirs[STEP_MAX_INST];
      int n = 0;
      for (int l = 1; l < L; ++l) {
        const int t = dg - (l - 1);
        if (t < 0 || t >= S) continue;
        LD& e = h->enc[l + 1];
        LstmFwdDir& d = dirs[n++];
        if (l == 1) {
          d.x = nullptr; d.ldx = 0; d.Kx = 0; d.gx = e.Gx + (size_t)t * Bp * 4 * H; d.ldgx = 4 * H; d.bias = nullptr;
        } else {
          d.x = drop ? h->enc[l].Yd + t * BP * esz : h->enc[l].Hst + (t + 1) * BP * esz;
          d.ldx = PH; d.Kx = H; d.gx = nullptr; d.ldgx = 0; d.bias = P + e.b_off;
        }
        d.hprev = e.Hst + t * BP * esz; d.ldh = e.ph;
        d.W = e.W; d.ldw = 2 * H; d.wx_off = 0; d.wh_off = H;
        d.cprev = e.Cst + t * BH; d.mask = h->mask_s + (size_t)t * Bp;
        d.hnext = e.Hst + (t + 1) * BP * esz; d.ldhn = e.ph; d.cnext = e.Cst + (t + 1) * BH;
        d.gsave = e.Gs + (size_t)t * Bp * 4 * H; d.ycat = nullptr; d.ldy = 0;
        if (drop && l + 1 < L) {
          d.ycat = e.Yd + t * BP * esz; d.ldy = e.ph; d.drop = drop_spec(h, DROP_SITE_ENC + l, t); d.drop_col0 = 0;
        }
        if (e.fm) {
          d.W_fm = e.Wfm; d.hprev_fm = e.HstF + t * BH * esz; d.hnext_fm = e.HstF + (t + 1) * BH * esz;
          if (l > 1) d.x_fm = drop ? h->enc[l].YdF + t * BH * esz : h->enc[l].HstF + (t + 1) * BH * esz;
          if (d.ycat) d.ycat_fm = e.YdF + t * BH * esz;
        }
      }
      launch_lstm_fwd(p, dirs, n, Bp, H, st);
    }
    Yprev = h->enc[L].Hst + BP * esz; ldY = PH;
  }
  const char* Hs = Yprev;
  const int ldHs = ldY;                          // source-side top-layer states [S, Bp, H]
  *Hs_out = Hs; *ldHs_out = ldHs;
  // attention keys K_i = W_a^T H_s^i for all i at once (Eq. 4 regrouped)
  launch_gemm_nt(p, Hs, ldHs, h->WaT, H, Ms, H, H, nullptr, h->Kmat, H, nullptr, 0, st);

  phase_mark(h, "keys, decoder init, decoder input GEMM");
  // ---- decoder initial state = encoder final state of the same depth ------------------------------
  {
    LD& d0 = h->dec[0];
    std::vector<CopyJob> cp;
    add_copy(cp, ef.Hst + (size_t)S * BPd * esz, ef.ph, d0.Hst, d0.ph, Bp, Hd, esz);
    add_copy(cp, eb.Hst, eb.ph, d0.Hst + (size_t)Hd * esz, d0.ph, Bp, Hd, esz);
    add_copy(cp, ef.Cst + (size_t)S * BHd, Hd, d0.Cst, H, Bp, Hd, 4);
    add_copy(cp, eb.Cst, Hd, d0.Cst + Hd, H, Bp, Hd, 4);
    for (int l = 1; l < L; ++l) {
      LD& e = h->enc[l + 1]; LD& d = h->dec[l];
      add_copy(cp, e.Hst + (size_t)S * BP * esz, e.ph, d.Hst, d.ph, Bp, H, esz);
      add_copy(cp, e.Cst + (size_t)S * BH, H, d.Cst, H, Bp, H, 4);
    }
    launch_copy2d_multi(cp.data(), (int)cp.size(), st);
    for (int l = 0; l < L; ++l)                     // fragment-major copies of the initial states
      if (h->dec[l].fm) launch_fm_pack(h->dec[l].Hst, h->dec[l].ph, Bp, H, h->dec[l].HstF, st);
  }
}

int enqueue_step(cmt_handle* h, const int32_t* src_ids, const int32_t* src_len, const int32_t* tgt_ids,
                 const int32_t* tgt_len, int B, int S, int T, bool forward_only) {
  const cmt_config& c = h->cfg;
  if (!src_ids || !src_len || !tgt_ids || !tgt_len) return fail(h, CMT_EINVAL, "null input pointer");
  if (B < 1 || B > c.max_batch || S < 1 || S > c.max_src_len || T < 1 || T > c.max_tgt_len)
    return fail(h, CMT_EINVAL, "B, S or T outside [1, configured maximum]");
  const int p = h->prec, E = c.emb_dim, H = c.hidden, Hd = H / 2, L = c.layers, V = c.tgt_vocab;
  const int Bp = round_up(B, 16);
  const size_t esz = h->esz;
  hipStream_t st = h->st;
  h->B = B; h->Bp = Bp; h->S = S; h->T = T;
  const int Ms = S * Bp, Mt = T * Bp;
  const size_t BH = (size_t)Bp * H;
  const int PH = h->PH;                            // row pitch of the H-wide per-step operands
  const bool drop = h->drop_p > 0.f;
  char* HoFeed = drop ? h->HoDrop : h->HoBuf;      // H_o as its consumers (output layer, input feed) see it
  const size_t BP = (size_t)Bp * PH;
  float* G = h->grads;
  float* P = h->params;

  h->phase_n = 0;
  phase_mark(h, "gathers + encoder bottom layer");
  {   // H_o^{<-1>} = 0, and the decoder's state gradients at the end of time = 0: one launch.  (The error flags
      // are not cleared here: they accumulate over the steps enqueued since the last read-back.)
    std::vector<FillJob> z;
    add_fill(z, h->HoBuf, BP, esz);
    if (drop) add_fill(z, h->HoDrop, BP, esz);
    if (h->HoFeedF) add_fill(z, h->HoFeedF, BH, esz);
    for (int l = 0; l < L; ++l) { add_fill(z, h->dec[l].dh, BH, 4); add_fill(z, h->dec[l].dc, BH, 4); }
    launch_fill_multi(z.data(), (int)z.size(), st);
  }
  // ---- embeddings, masks ------------------------------------------------------------------------
  launch_gather(p, h->Pw(h->off_Esrc), c.src_vocab, E, src_ids, src_len, B, Bp, S, 0, 0, h->Xs, h->mask_s, h->tok_s,
                nullptr, h->len_s, h->flags, st);
  launch_gather(p, h->Pw(h->off_Etgt), c.tgt_vocab, E, tgt_ids, tgt_len, B, Bp, T, 1, c.bos_id, h->Xt, h->mask_t,
                h->tok_t, h->labels, h->len_t, h->flags, st);
  // valid target positions numbered densely, n_tok, 1 / n_tok: the lengths give them
  launch_ce_compact(h->mask_t, h->labels, Mt, h->ce_pos, h->ce_row, h->labels_c, h->rowscale, h->ce_nvalid, h->loss, st);

  const char* Hs; int ldHs;                        // source-side top-layer states [S, Bp, H] and their row pitch
  enqueue_encoder(h, S, &Hs, &ldHs);
  LD& ef = h->enc[0]; LD& eb = h->enc[1];
  const size_t BHd = (size_t)Bp * Hd;
  // ---- decoder time loop --------------------------------------------------------------------------
  // The attentional layer's pre-activation W_c [C_s; H_t] (Eq. 7) is sum_i a_i (W_c1 H_s^i) + W_c2 H_t: with the rows
  // W_c1 H_s^i made once per batch, a step needs no context before its H_o, and the W_c2 H_t sums share a launch
  // with the scores (both wait for the top layer's state alone) — two dependent launches per step instead of three.
  // The contexts themselves (the weight gradient of W_c needs them) are made for all steps at once afterwards.
  const bool proj = h->att_proj && Bp < 256;
  {
    LD& d0 = h->dec[0];
    launch_gemm_nt(p, h->Xt, E, d0.W, E + 2 * H, Mt, 4 * H, E, d0.Gx, nullptr, 4 * H, P + d0.b_off, 0, st);
    if (proj) launch_gemm_nt(p, Hs, ldHs, h->Pw(h->off_Wc), 2 * H, Ms, H, H, h->Pmat, h->PmatT, H, nullptr, 0, st);
    phase_mark(h, "decoder forward loop");
    for (int j = 0; j < T; ++j) {
      for (int l = 0; l < L; ++l) dec_lstm_fwd(h, l, j);
      const char* Ht = h->dec[L - 1].Hst + (j + 1) * BP * esz;
      if (proj) { dec_att_fwd_proj(h, j, S, h->att_s + (size_t)j * Bp * S); continue; }
      StepGemm g{};
      g.a0 = h->Cs + j * BP * esz; g.lda0 = PH; g.K0 = H; g.w0_off = 0;
      g.a1 = Ht; g.lda1 = PH; g.K1 = H; g.w1_off = H;
      g.W = h->Pw(h->off_Wc); g.ldw = 2 * H; g.N = H; g.mode = 0;
      g.out = h->wcp; g.ldout = H; g.plane_stride = BH;
      launch_att_fwd(p, h->Kmat, H, Hs, ldHs, Ht, PH, h->len_s, S, Bp, H, h->att_s + (size_t)j * Bp * S,
                     h->att_a + (size_t)j * Bp * S, h->Cs + j * BP * esz, PH, st, h->CsF ? h->CsF + j * BH * esz : nullptr);
      g.outT = h->HoBuf + (j + 1) * BP * esz; g.ldo = PH;
      if (drop) { g.outD = h->HoDrop + (j + 1) * BP * esz; g.ldod = PH; g.drop = drop_spec(h, DROP_SITE_HO, j); }
      if (h->HoFeedF) {
        g.outF = h->HoFeedF + (j + 1) * BH * esz;
        g.W_fm = h->WcF; g.a0_fm = h->CsF + j * BH * esz; g.a1_fm = h->dec[L - 1].HstF + (j + 1) * BH * esz;
      }
      launch_step_gemm(p, g, Bp, st);
    }
  }
  phase_mark(h, "output layer forward + backward");
  // =================================== output layer (Eq. 1) and backward ==============================
  // The recurrences' backward loops are chains of short dependent kernels that leave most of the
  // chip idle; everything that does not feed them (transposes, weight gradients, dW_o, embedding
  // scatters) runs on the library's second stream and joins at the end of the step.
  const char* Ho = HoFeed + BP * esz;              // [T*Bp, H], row pitch PH
  const int np = ce_num_partials(V);
  // The output layer sees the valid target positions only: their H_o rows are gathered into a dense
  // matrix (the count is known to the device alone, so launches are sized for all T * Bp rows and the
  // kernels stop at the count).
  launch_ce_gather_rows(p, Ho, PH, h->ce_row, h->ce_nvalid, Mt, h->Hoc, PH, H, st);
  if (forward_only) {                              // Eq. 1 and the loss only: logits slab by slab, no gradient
    if (proj) launch_att_context(p, Hs, ldHs, h->att_a, h->len_s, S, T, Bp, H, h->Cs, PH, st);   // (for the read-back by name)
    int nslab;
    const int rows = ce_slab_plan(h, Mt, &nslab);
    int sl = 0;
    for (int m0 = 0; m0 < Mt; ++sl) {
      const int Mc = (sl == nslab - 1 || Mt - m0 < rows) ? Mt - m0 : rows;
      const RowLimit lim{h->ce_nvalid, m0};
      const size_t po = (size_t)sl * np * h->ce_pitch;       // this slab's block of partials
      launch_ce_fwd(p, h->Hoc + (size_t)m0 * PH * esz, PH, h->Pw(h->off_Wo), P + h->off_Bo, h->labels_c + m0, Mc, V, H, h->dzTs,
                    h->ce_pitch, h->pmax + po, h->psum + po, h->ls_eps > 0.f ? h->psz + po : nullptr, h->zy + m0, st, lim);
      launch_ce_rows(h->pmax + po, h->psum + po, h->psz + po, h->zy + m0, nullptr, Mc, np, h->ce_pitch, h->ls_eps, V,
                     h->lse + m0, h->nll + m0, st, lim);
      m0 += Mc;
    }
    launch_ce_loss(h->nll, Mt, h->loss, h->flags, st, RowLimit{h->ce_nvalid, 0});
    phase_mark(h, "end");
    (void)hipMemcpyAsync(h->h_loss, h->loss, 2 * sizeof(float), hipMemcpyDeviceToHost, st);
    (void)hipMemcpyAsync(h->h_flags, h->flags, sizeof(int), hipMemcpyDeviceToHost, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e, "enqueue");
    h->have_step = true;
    return CMT_OK;
  }
  hipStream_t sd = h->use_side ? h->side : st;
  const int ldHoT = Mt + Bp;
  auto transpose_states = [&](LD& d, int Lsteps) {
    launch_transpose(p, d.Hst, d.ph, d.HstT, (Lsteps + 1) * Bp, (Lsteps + 1) * Bp, d.Hh, sd);
  };
  stream_after(h, sd, st);
  // the dense embedding gradients start from zero: cleared now, while the second stream has little to do
  launch_fill_f32(G + h->off_Esrc, (size_t)c.src_vocab * E, 0.f, sd);
  launch_fill_f32(G + h->off_Etgt, (size_t)c.tgt_vocab * E, 0.f, sd);
  hipEvent_t esrc_cleared = nullptr;               // the source table's scatter runs on the caller's stream at the end
  if (sd != st) {
    esrc_cleared = h->ev[h->ev_next++ % h->ev.size()];
    (void)hipEventRecord(esrc_cleared, sd);
  }
  launch_transpose(p, h->Hoc, PH, h->HocT, Mt, Mt, H, sd);           // dense H_o rows, for dW_o
  launch_transpose(p, HoFeed, PH, h->HoBufT, ldHoT, Mt + Bp, H, sd);
  for (auto& d : h->enc) transpose_states(d, S);
  for (auto& d : h->dec) transpose_states(d, T);
  if (drop) {                                      // inputs of the layers above, as they saw them
    for (int l = 1; l + 1 < L; ++l) launch_transpose(p, h->enc[l + 1].Yd, PH, h->enc[l + 1].YdT, Ms, Ms, H, sd);
    for (int l = 0; l + 1 < L; ++l) launch_transpose(p, h->dec[l].Yd, PH, h->dec[l].YdT, Mt, Mt, H, sd);
  }
  launch_transpose(p, h->Y0, H, h->Y0T, Ms, Ms, H, sd);
  launch_transpose(p, h->Xs, E, h->XsT, Ms, Ms, E, sd);
  launch_transpose(p, h->Xt, E, h->XtT, Mt, Mt, E, sd);
  if (proj) launch_att_context(p, Hs, ldHs, h->att_a, h->len_s, S, T, Bp, H, h->Cs, PH, sd);
  launch_transpose(p, h->Cs, PH, h->CsT, Mt, Mt, H, sd);
  {
    // Full slabs of the slab capacity and one remainder (one slab whenever the batch fits), two slab buffer pairs, over the dense rows of
    // the valid target positions.  The host sizes the slabs for all T * Bp rows; every kernel gets the
    // device's count and a slab that lies beyond it costs a few empty launches.  Per slab the main
    // stream takes forward (logits -> e, partials), lse / nll, e -> dz and dz^T, and dH_o = dz W_o (the
    // decoder needs it); the second stream takes dW_o += dz^T H_o and dB_o.
    int nslab;
    const int rows = ce_slab_plan(h, Mt, &nslab);
    std::vector<hipEvent_t> done(nslab, nullptr);
    const float eps = h->ls_eps;
    int sl = 0, n_dbo = 0;
    for (int m0 = 0; m0 < Mt; ++sl) {
      const int Mc = (sl == nslab - 1 || Mt - m0 < rows) ? Mt - m0 : rows;
      const RowLimit lim{h->ce_nvalid, m0};
      char* dz = (sl & 1) ? h->dzs2 : h->dzs;
      char* dzT = (sl & 1) ? h->dzTs2 : h->dzTs;
      if (sl >= 2 && sd != st) (void)hipStreamWaitEvent(st, done[sl - 2], 0);
      const size_t po = (size_t)sl * np * h->ce_pitch;       // this slab's block of partials
      launch_ce_fwd(p, h->Hoc + (size_t)m0 * PH * esz, PH, h->Pw(h->off_Wo), P + h->off_Bo, h->labels_c + m0, Mc, V, H, dzT,
                    h->ce_pitch, h->pmax + po, h->psum + po, eps > 0.f ? h->psz + po : nullptr, h->zy + m0, st, lim);
      launch_ce_rows(h->pmax + po, h->psum + po, h->psz + po, h->zy + m0, nullptr, Mc, np, h->ce_pitch, eps, V, h->lse + m0,
                     h->nll + m0, st, lim);
      launch_ce_scale(p, dzT, h->ce_pitch, V, Mc, h->pmax + po, h->lse + m0, h->labels_c + m0, h->rowscale + m0, eps, dz,
                      h->dbo_parts + (size_t)n_dbo * V, st, lim);
      n_dbo += (Mc + 63) / 64;
      stream_after(h, sd, st);
      launch_gemm_nt(p, dz, V, h->WoT, V, Mc, H, V, h->dHoCE + (size_t)m0 * H, nullptr, H, nullptr, 0, st, h->gsplit,
                     h->gsplit_floats, lim, 1);                           // dH_o[slab] = dz W_o
      // dW_o (+)= dz^T H_o[slab]; the first slab always holds a row, so W_o's gradient is always written
      launch_gemm_nt(p, dzT, h->ce_pitch, h->HocT + (size_t)m0 * esz, Mt, V, H, Mc, G + h->off_Wo, nullptr, H, nullptr, sl > 0,
                     sd, nullptr, 0, lim, 2, sd != st ? h->side_cap(h->side_wgs_wo) : 0);
      if (sd != st) {
        done[sl] = h->ev[h->ev_next++ % h->ev.size()];
        (void)hipEventRecord(done[sl], sd);
      }
      m0 += Mc;
    }
    launch_sum_parts(h->dbo_parts, n_dbo, (size_t)V, G + h->off_Bo, st);
    launch_ce_loss(h->nll, Mt, h->loss, h->flags, st, RowLimit{h->ce_nvalid, 0});
  }

  phase_mark(h, "decoder backward loop");
  // ---- decoder loop backwards -----------------------------------------------------------------------
  const int kbd = step_kblocks(p, 2 * H, 4 * H, Bp, h->kb_bwd_dec);       // planes written by a decoder layer's backward GEMM
  const size_t pstr = (size_t)Bp * 2 * H;
  const Planes no_planes{nullptr, 0, 0, 0};
  if ((h->bwd_fused & 1) && Bp <= 128) {            // (measured at 128 sentences: 8.1 against 8.7 ms for the k-split form)
    // one launch per layer and step (dec_bwd_gemm): no pointwise launches, no planes
    for (int j = T - 1; j >= 0; --j) {
      char* dpre = h->dPre + j * BP * esz;
      const bool last = j == T - 1;
      char* dpreF = h->dPreF ? h->dPreF + j * BH * esz : nullptr;
      if (last)
        launch_tanh_bwd(p, h->dHoCE, h->ce_pos + (size_t)j * Bp, no_planes, h->HoBuf + (j + 1) * BP * esz, PH, dpre, PH, Bp, H,
                        drop_spec(h, DROP_SITE_HO, j), st, dpreF);
      int kbw = step_kblocks(p, 2 * H, H, Bp, h->kb_wc);
      if (proj && (h->att_proj & 1) && h->wc_whole_k) {
        dec_att_bwd_proj(h, j, S, last);
        for (int l = L - 1; l >= 0; --l) {
          const StepBwd gl = dec_bwd_gemm(h, l, j);
          launch_step_bwd_fused(p, &gl, 1, Bp, st);
        }
        continue;
      }
      if (h->wc_whole_k) {   // [dC_s ; dH_t] = dpre W_c with the whole (short) k range per workgroup: one plane
        StepBwd g{};
        g.dg = dpre; g.lddg = PH; g.K = H; g.Wt = h->WcT; g.ldw = H;
        g.part[0].kind = BWD_EPI_STORE; g.part[0].ncols = 2 * H; g.part[0].out = h->wcp; g.part[0].ldout = 2 * H;
        g.dg_fm = dpreF; g.Wt_fm = dpreF ? h->WcTF : nullptr; g.wt_tile0 = 0;
        launch_step_bwd_fused(p, &g, 1, Bp, st);
        kbw = 1;
      } else {   // the same as k blocks into planes
        StepGemm g{};
        g.a0 = dpre; g.lda0 = PH; g.K0 = H; g.w0_off = 0; g.K1 = 0;
        g.W = h->WcT; g.ldw = H; g.N = 2 * H; g.mode = 1; g.max_kb = h->kb_wc;
        g.out = h->wcp; g.ldout = 2 * H; g.plane_stride = pstr;
        g.W_fm = h->WcTF; g.a0_fm = dpreF;
        launch_step_gemm(p, g, Bp, st);
      }
      // attention backward; the gradient it sends to the top layer's output stays in registers and that
      // layer's cell backward runs in the same launch
      LstmBwdPoint top = dec_cell(h, L - 1, j);
      top.dhrec = Planes{h->dec[L - 1].bwdp, H, last ? 0 : 1, 0};
      launch_att_bwd(p, h->Kmat, H, Hs, ldHs, Planes{h->wcp, 2 * H, kbw, pstr}, h->dCs + j * BH, h->att_a + (size_t)j * Bp * S,
                     h->len_s, S, Bp, H, h->dots, h->att_ds + (size_t)j * Bp * S, h->dHt, st, &top);
      for (int l = L - 1; l >= 0; --l) {
        const StepBwd g = dec_bwd_gemm(h, l, j);
        launch_step_bwd_fused(p, &g, 1, Bp, st);
      }
    }
    for (int l = 0; l < L; ++l)
      launch_planes_add(h->dec[l].dh, h->dec[l].dh, Planes{h->dec[l].bwdp, H, 1, 0}, 0, Bp, H, st);
  } else {
  for (int j = T - 1; j >= 0; --j) {
    char* dpre = h->dPre + j * BP * esz;
    const bool last = j == T - 1;
    // dH_o = cross-entropy part + what step j+1's bottom layer sent back through the input feed
    char* dpreF = h->dPreF ? h->dPreF + j * BH * esz : nullptr;
    launch_tanh_bwd(p, h->dHoCE, h->ce_pos + (size_t)j * Bp, Planes{h->dec[0].bwdp, 2 * H, last ? 0 : kbd, pstr}, h->HoBuf + (j + 1) * BP * esz,
                    PH, dpre, PH, Bp, H, drop_spec(h, DROP_SITE_HO, j), st, dpreF);
    const int kbw = step_kblocks(p, 2 * H, H, Bp, h->kb_wc);
    {   // [dC_s ; dH_t] = dpre W_c, as planes
      StepGemm g{};
      g.a0 = dpre; g.lda0 = PH; g.K0 = H; g.w0_off = 0; g.K1 = 0;
      g.W = h->WcT; g.ldw = H; g.N = 2 * H; g.mode = 1; g.max_kb = h->kb_wc;
      g.out = h->wcp; g.ldout = 2 * H; g.plane_stride = pstr;
      g.W_fm = h->WcTF; g.a0_fm = dpreF;
      launch_step_gemm(p, g, Bp, st);
    }
    launch_att_bwd(p, h->Kmat, H, Hs, ldHs, Planes{h->wcp, 2 * H, kbw, pstr}, h->dCs + j * BH, h->att_a + (size_t)j * Bp * S,
                   h->len_s, S, Bp, H, h->dots, h->att_ds + (size_t)j * Bp * S, h->dHt, st);
    for (int l = L - 1; l >= 0; --l) {
      LD& e = h->dec[l];
      LstmBwdPoint q;
      if (l == L - 1) q.dy = Planes{h->dHt, H, 1, 0};
      else { q.dy = Planes{h->dec[l + 1].bwdp, 2 * H, kbd, pstr}; q.drop_dy = drop_spec(h, DROP_SITE_DEC + l, j); }
      q.dy_col = 0;                                                   // dx of the layer above, columns [0, H)
      q.dhrec = Planes{e.bwdp, 2 * H, last ? 0 : kbd, pstr}; q.dhrec_col = H;
      q.dh = e.dh; q.dc = e.dc;
      q.gsave = e.Gs + (size_t)j * Bp * 4 * H;
      q.cprev = e.Cst + j * BH; q.cnext = e.Cst + (j + 1) * BH;
      q.mask = h->mask_t + (size_t)j * Bp;
      q.dg = e.dG + (size_t)j * Bp * e.pg * esz; q.lddg = e.pg;
      if (e.fmb) q.dg_fm = e.dGF + (size_t)j * Bp * 4 * H * esz;
      launch_lstm_bwd_point(p, q, Bp, H, st);
      StepGemm g{};                                  // [dx ; dh_prev] = dgates [W_x ; W_h] (bottom layer: [feed ; h])
      g.a0 = q.dg; g.lda0 = e.pg; g.K0 = 4 * H; g.w0_off = 0; g.K1 = 0;
      g.W = e.Wt + (size_t)(l == 0 ? E : 0) * 4 * H * esz; g.ldw = 4 * H;
      if (e.fmb) { g.W_fm = e.WtF; g.w_tile0 = (l == 0 ? E : 0) / 16; g.a0_fm = q.dg_fm; }
      g.N = 2 * H; g.mode = 1; g.max_kb = h->kb_bwd_dec;
      g.out = e.bwdp; g.ldout = 2 * H; g.plane_stride = pstr;
      launch_step_gemm(p, g, Bp, st);
    }
  }
  // gradient of the decoder's initial state: pass-through part + the last GEMM's recurrent part
  for (int l = 0; l < L; ++l)
    launch_planes_add(h->dec[l].dh, h->dec[l].dh, Planes{h->dec[l].bwdp, 2 * H, kbd, pstr}, H, Bp, H, st);
  }

  phase_mark(h, "deferred attention gradients");
  // ---- second stream: everything that only needed the decoder's dgates and dpre -----------------------
  stream_after(h, sd, st);
  launch_transpose(p, h->dPre, PH, h->dPreT, Mt, Mt, H, sd);
  // encoder layer outputs, transposed: layer 0 -> Y0T (ld Ms); layer l >= 1 -> HstT + Bp (ld (S+1)Bp)
  auto encYT = [&](int l, int* ld) -> const char* {
    if (l == 0) { *ld = Ms; return h->Y0T; }
    if (drop && l + 1 < L) { *ld = Ms; return h->enc[l + 1].YdT; }
    *ld = (S + 1) * Bp; return h->enc[l + 1].HstT + (size_t)Bp * esz;
  };
  // dW_c = dpre^T [C_s ; H_t]
  h->dw_group.push_back(GemmProb{h->dPreT, h->CsT, G + h->off_Wc, Mt, Mt, 2 * H, H, H, Mt, 0});
  h->dw_group.push_back(GemmProb{h->dPreT, h->dec[L - 1].HstT + (size_t)Bp * esz, G + h->off_Wc + H, Mt, (T + 1) * Bp, 2 * H, H, H, Mt, 0});
  for (int l = 0; l < L; ++l) {
    LD& e = h->dec[l];
    if (l == 0)
      weight_grads(h, e, T, {{h->XtT, Mt}, {h->HoBufT, ldHoT}, {e.HstT, (T + 1) * Bp}}, {E, H, H}, sd);
    else
      weight_grads(h, e, T, {drop ? std::pair<const char*, int>{h->dec[l - 1].YdT, Mt}
                                  : std::pair<const char*, int>{h->dec[l - 1].HstT + (size_t)Bp * esz, (T + 1) * Bp},
                             {e.HstT, (T + 1) * Bp}}, {H, H}, sd);
  }
  flush_dw_group(h, sd);                           // W_c and every decoder layer's weight gradient: one launch
  launch_gemm_nt(p, h->dec[0].dG, h->dec[0].pg, h->dec[0].Wt, 4 * H, Mt, E, 4 * H, h->dXt, nullptr, E, nullptr, 0, sd);
  launch_embed_scatter(h->dXt, h->tok_t, Mt, c.tgt_vocab, E, G + h->off_Etgt, sd, false);

  // ---- attention gradients that do not feed the decoder recurrence, batched over all steps ---------
  const char* HtAll = h->dec[L - 1].Hst + BP * esz;      // H_t^{<0..T-1>}
  launch_att_deferred(p, h->att_a, h->att_ds, h->dCs, H, HtAll, PH, S, T, Bp, H, h->dHs, h->dK, st);
  launch_gemm_nt(p, h->dK, H, h->Pw(h->off_Wa), H, Ms, H, H, h->dHs, nullptr, H, nullptr, 1, st);   // dHs += dK W_a^T
  stream_after(h, sd, st);
  launch_transpose(p, h->dK, H, h->dKT, Ms, Ms, H, sd);
  {   // dW_a[r,c] = sum_i H_s[i,r] dK[i,c]
    int ld; const char* HsT = encYT(L - 1, &ld);
    h->dw_group.push_back(GemmProb{HsT, h->dKT, G + h->off_Wa, ld, Ms, H, H, H, Ms, 0});
    flush_dw_group(h, sd);
  }

  phase_mark(h, "encoder upper layers backward");
  // ---- encoder backwards ------------------------------------------------------------------------------
  // Upper layers: the same wavefront, top layer first.  Per diagonal one pointwise launch (cell
  // backward of every active layer-step) and one step-GEMM launch ([dx; dh_prev] = dgates [W_x; W_h]).
  const bool upper_fused = h->bwd_fused_auto ? (double)(L - 1) * Bp * H * H <= 134217728.0 : (h->bwd_fused & 2) != 0;
  if (L > 1 && upper_fused) {
    // Fused form: one launch per diagonal.  The step GEMM of (layer l, position t) keeps its dh_prev half in
    // registers and runs the cell backward of (l, t - 1) in its epilogue; its dx half is stored for the layer
    // below (two alternating slots of bwdp per layer, Bp * H floats each).  Layer l at position t - 1 needs the
    // dx of layer l + 1 at t - 1 from an earlier launch, so a layer runs two diagonals behind the one above:
    // (l, t) sits on diagonal (S - 1 - t) + 2 (L - 1 - l).  The first position of a layer has no GEMM
    // before it: its cell backward is a pointwise launch just ahead of the layer's first diagonal.
    const size_t slot = (size_t)Bp * H;
    auto enc_cell = [&](int l, int t) {
      LD& e = h->enc[l + 1];
      LstmBwdPoint q;
      if (l == L - 1) q.dy = Planes{h->dHs + (size_t)t * Bp * H, H, 1, 0};
      else { q.dy = Planes{h->enc[l + 2].bwdp + (size_t)(t & 1) * slot, H, 1, 0}; q.drop_dy = drop_spec(h, DROP_SITE_ENC + l, t); }
      q.dy_col = 0;
      q.dhrec = Planes{nullptr, 0, 0, 0}; q.dhrec_col = 0;
      q.dh = h->dec[l].dh; q.dc = h->dec[l].dc;      // gradient of the final state = gradient of the decoder's initial state
      q.gsave = e.Gs + (size_t)t * Bp * 4 * H;
      q.cprev = e.Cst + t * BH; q.cnext = e.Cst + (t + 1) * BH;
      q.mask = h->mask_s + (size_t)t * Bp;
      q.dg = e.dG + (size_t)t * Bp * e.pg * esz; q.lddg = e.pg;
      if (e.fmb) q.dg_fm = e.dGF + (size_t)t * Bp * 4 * H * esz;
      return q;
    };
    for (int dg = 0; dg <= (S - 1) + 2 * (L - 2); ++dg) {
      StepBwd gs[STEP_MAX_INST];
      int ng = 0;
      for (int l = L - 1; l >= 1; --l) {
        const int k = dg - 2 * (L - 1 - l);
        if (k < 0 || k >= S) continue;
        const int t = S - 1 - k;
        LD& e = h->enc[l + 1];
        if (k == 0) launch_lstm_bwd_point(p, enc_cell(l, t), Bp, H, st);
        if (l == 1 && t == 0) continue;              // the initial state is a constant, and layer 1's dx is batched below
        StepBwd& g = gs[ng++];
        g = StepBwd{};
        g.dg = e.dG + (size_t)t * Bp * e.pg * esz; g.lddg = e.pg; g.K = 4 * H; g.ldw = 4 * H;
        int np = 0;
        if (l > 1) {
          g.Wt = e.Wt;
          BwdEpi& d = g.part[np++];
          d.kind = BWD_EPI_STORE; d.ncols = H; d.hh = H; d.out = e.bwdp + (size_t)(t & 1) * slot; d.ldout = H;
        } else {
          g.Wt = e.Wt + (size_t)H * 4 * H * esz;
        }
        if (e.fmb) { g.dg_fm = e.dGF + (size_t)t * Bp * 4 * H * esz; g.Wt_fm = e.WtF; g.wt_tile0 = (l > 1 ? 0 : H) / 16; }
        if (t > 0) {
          BwdEpi& r = g.part[np++];
          r.kind = BWD_EPI_CELL_REC; r.ncols = H; r.hh = H; r.cell = enc_cell(l, t - 1);
        }
      }
      if (ng) launch_step_bwd_fused(p, gs, ng, Bp, st);
    }
    LD& e1 = h->enc[2];
    launch_gemm_nt(p, e1.dG, e1.pg, e1.Wt, 4 * H, Ms, H, 4 * H, h->dYa, nullptr, H, nullptr, 0, st);   // layer 0's dY = dG_1 W_x
    stream_after(h, sd, st);
    for (int l = L - 1; l >= 1; --l) {
      LD& e = h->enc[l + 1];
      int ld; const char* XT = encYT(l - 1, &ld);
      weight_grads(h, e, S, {{XT, ld}, {e.HstT, (S + 1) * Bp}}, {H, H}, sd);
    }
    flush_dw_group(h, sd);
  } else if (L > 1) {
    const int Nplan = L > 2 ? 2 * H : H;
    const int kbE = step_kblocks(p, Nplan, 4 * H, Bp, h->kb_bwd);
    const size_t pstrE = (size_t)Bp * 2 * H;
    for (int dg = 0; dg < S + L - 2; ++dg) {
      LstmBwdPoint pts[STEP_MAX_INST];
      StepGemm gs[STEP_MAX_INST];
      int n = 0, ng = 0;
      for (int l = L - 1; l >= 1; --l) {
        const int k = dg - (L - 1 - l);
        if (k < 0 || k >= S) continue;
        const int t = S - 1 - k;
        LD& e = h->enc[l + 1];
        LstmBwdPoint& q = pts[n++];
        if (l == L - 1) q.dy = Planes{h->dHs + (size_t)t * Bp * H, H, 1, 0};
        else { q.dy = Planes{h->enc[l + 2].bwdp, 2 * H, kbE, pstrE}; q.drop_dy = drop_spec(h, DROP_SITE_ENC + l, t); }
        q.dy_col = 0;                                                       // dx of the layer above (its columns [0, H))
        q.dhrec = Planes{e.bwdp, 2 * H, k == 0 ? 0 : kbE, pstrE};
        q.dhrec_col = (l == 1) ? 0 : H;                                     // layer 1 only computes the recurrent part
        // gradient of the final state = gradient of the decoder's initial state of the same depth
        q.dh = h->dec[l].dh; q.dc = h->dec[l].dc;
        q.gsave = e.Gs + (size_t)t * Bp * 4 * H;
        q.cprev = e.Cst + t * BH; q.cnext = e.Cst + (t + 1) * BH;
        q.mask = h->mask_s + (size_t)t * Bp;
        q.dg = e.dG + (size_t)t * Bp * e.pg * esz; q.lddg = e.pg;
        if (e.fmb) q.dg_fm = e.dGF + (size_t)t * Bp * 4 * H * esz;
        if (l == 1 && k == S - 1) continue;                                 // the initial state is a constant
        StepGemm& g = gs[ng++];
        g = StepGemm{};
        g.a0 = q.dg; g.lda0 = e.pg; g.K0 = 4 * H; g.w0_off = 0; g.K1 = 0;
        g.W = e.Wt + (size_t)(l == 1 ? H : 0) * 4 * H * esz; g.ldw = 4 * H;
        if (e.fmb) { g.W_fm = e.WtF; g.w_tile0 = (l == 1 ? H : 0) / 16; g.a0_fm = q.dg_fm; }
        g.N = (l == 1) ? H : 2 * H; g.mode = 1; g.max_kb = h->kb_bwd;
        g.out = e.bwdp; g.ldout = 2 * H; g.plane_stride = pstrE;
      }
      launch_lstm_bwd_point_multi(p, pts, n, Bp, H, st);
      if (ng) launch_step_gemm_multi(p, gs, ng, Nplan, Bp, st);
    }
    LD& e1 = h->enc[2];
    launch_gemm_nt(p, e1.dG, e1.pg, e1.Wt, 4 * H, Ms, H, 4 * H, h->dYa, nullptr, H, nullptr, 0, st);   // layer 0's dY = dG_1 W_x
    stream_after(h, sd, st);
    for (int l = L - 1; l >= 1; --l) {
      LD& e = h->enc[l + 1];
      int ld; const char* XT = encYT(l - 1, &ld);
      weight_grads(h, e, S, {{XT, ld}, {e.HstT, (S + 1) * Bp}}, {H, H}, sd);
    }
    flush_dw_group(h, sd);
  }
  phase_mark(h, "encoder bottom layer backward");
  {   // bottom layer: the two directions run in the same launches
    const float* dY0 = L > 1 ? h->dYa : h->dHs;
    LD& d0 = h->dec[0];
    std::vector<CopyJob> cp;
    add_copy(cp, d0.dh, H, ef.dh, Hd, Bp, Hd, 4); add_copy(cp, d0.dh + Hd, H, eb.dh, Hd, Bp, Hd, 4);
    add_copy(cp, d0.dc, H, ef.dc, Hd, Bp, Hd, 4); add_copy(cp, d0.dc + Hd, H, eb.dc, Hd, Bp, Hd, 4);
    launch_copy2d_multi(cp.data(), (int)cp.size(), st);
    const int kb0 = step_kblocks(p, Hd, 4 * Hd, Bp, h->kb_bwd);
    const size_t pstr0 = (size_t)Bp * Hd;
    // cell backward of direction i at position t (its dy is a slice of the batched dY of the layer above)
    auto enc0_cell = [&](int i, int t) {
      LD& e = i ? eb : ef;
      const int slot_prev = i ? t + 1 : t, slot_next = i ? t : t + 1;
      LstmBwdPoint q;
      q.dy = Planes{dY0 + (size_t)t * Bp * H, H, 1, 0}; q.dy_col = i ? Hd : 0;
      if (L > 1) q.drop_dy = drop_spec(h, DROP_SITE_ENC + 0, t);
      q.dhrec = Planes{nullptr, 0, 0, 0}; q.dhrec_col = 0;
      q.dh = e.dh; q.dc = e.dc;
      q.gsave = e.Gs + (size_t)t * Bp * 4 * Hd;
      q.cprev = e.Cst + (size_t)slot_prev * BHd; q.cnext = e.Cst + (size_t)slot_next * BHd;
      q.mask = h->mask_s + (size_t)t * Bp;
      q.dg = e.dG + (size_t)t * Bp * e.pg * esz; q.lddg = e.pg;
      if (e.fmb) q.dg_fm = e.dGF + (size_t)t * Bp * 4 * Hd * esz;
      return q;
    };
    if (h->bwd_fused & 4) {
      // one launch per position: dh_prev = dgates W_h of both directions, the cell backward of each
      // direction's next position in the epilogue; only the very first position is a pointwise launch
      LstmBwdPoint first[2] = {enc0_cell(0, S - 1), enc0_cell(1, 0)};
      launch_lstm_bwd_point_multi(p, first, 2, Bp, Hd, st);
      for (int k = 0; k + 1 < S; ++k) {
        StepBwd gs[2];
        for (int i = 0; i < 2; ++i) {
          LD& e = i ? eb : ef;
          const int t = i ? k : S - 1 - k, tn = i ? k + 1 : S - 2 - k;
          StepBwd& g = gs[i];
          g = StepBwd{};
          g.dg = e.dG + (size_t)t * Bp * e.pg * esz; g.lddg = e.pg; g.K = 4 * Hd;
          g.Wt = e.Wt + (size_t)E * 4 * Hd * esz; g.ldw = 4 * Hd;
          if (e.fmb) { g.dg_fm = e.dGF + (size_t)t * Bp * 4 * Hd * esz; g.Wt_fm = e.WtF; g.wt_tile0 = E / 16; }
          BwdEpi& r = g.part[0];
          r.kind = BWD_EPI_CELL_REC; r.ncols = Hd; r.hh = Hd; r.cell = enc0_cell(i, tn);
        }
        launch_step_bwd_fused(p, gs, 2, Bp, st);
      }
    } else
    for (int k = 0; k < S; ++k) {
      LstmBwdPoint pts[2];
      StepGemm gs[2];
      for (int i = 0; i < 2; ++i) {
        LD& e = i ? eb : ef;
        const int t = i ? k : S - 1 - k;                                    // reverse of each direction's processing order
        const int slot_prev = i ? t + 1 : t, slot_next = i ? t : t + 1;
        LstmBwdPoint& q = pts[i];
        q.dy = Planes{dY0 + (size_t)t * Bp * H, H, 1, 0}; q.dy_col = i ? Hd : 0;
        if (L > 1) q.drop_dy = drop_spec(h, DROP_SITE_ENC + 0, t);
        q.dhrec = Planes{e.bwdp, Hd, k == 0 ? 0 : kb0, pstr0}; q.dhrec_col = 0;
        q.dh = e.dh; q.dc = e.dc;
        q.gsave = e.Gs + (size_t)t * Bp * 4 * Hd;
        q.cprev = e.Cst + (size_t)slot_prev * BHd; q.cnext = e.Cst + (size_t)slot_next * BHd;
        q.mask = h->mask_s + (size_t)t * Bp;
        q.dg = e.dG + (size_t)t * Bp * e.pg * esz; q.lddg = e.pg;
        StepGemm& g = gs[i];
        g = StepGemm{};
        g.a0 = q.dg; g.lda0 = e.pg; g.K0 = 4 * Hd; g.w0_off = 0; g.K1 = 0;
        g.W = e.Wt + (size_t)E * 4 * Hd * esz; g.ldw = 4 * Hd;
        g.N = Hd; g.mode = 1; g.max_kb = h->kb_bwd;
        g.out = e.bwdp; g.ldout = Hd; g.plane_stride = pstr0;
      }
      launch_lstm_bwd_point_multi(p, pts, 2, Bp, Hd, st);
      if (k + 1 < S) launch_step_gemm_multi(p, gs, 2, Hd, Bp, st);          // the initial state is a constant
    }
    // What is left after the last recurrent kernel is shared between the two streams: the weight gradients of
    // both directions on the second one, the source-embedding gradient (dX_s, then the scatter) on the caller's.
    stream_after(h, sd, st);
    weight_grads(h, ef, S, {{h->XsT, Ms}, {ef.HstT, (S + 1) * Bp}}, {E, Hd}, sd);
    weight_grads(h, eb, S, {{h->XsT, Ms}, {eb.HstT + (size_t)Bp * esz, (S + 1) * Bp}}, {E, Hd}, sd);
    flush_dw_group(h, sd);
    launch_gemm_nt(p, ef.dG, ef.pg, ef.Wt, 4 * Hd, Ms, E, 4 * Hd, h->dXs, nullptr, E, nullptr, 0, st);
    launch_gemm_nt(p, eb.dG, eb.pg, eb.Wt, 4 * Hd, Ms, E, 4 * Hd, h->dXs, nullptr, E, nullptr, 1, st);
    if (esrc_cleared) (void)hipStreamWaitEvent(st, esrc_cleared, 0);
    launch_embed_scatter(h->dXs, h->tok_s, Ms, c.src_vocab, E, G + h->off_Esrc, st, false);
  }
  phase_mark(h, "wait for the second stream");
  stream_after(h, st, sd);                         // join: the step is complete on the caller's stream
  phase_mark(h, "end");
  (void)hipMemcpyAsync(h->h_loss, h->loss, 2 * sizeof(float), hipMemcpyDeviceToHost, st);
  (void)hipMemcpyAsync(h->h_flags, h->flags, sizeof(int), hipMemcpyDeviceToHost, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "enqueue");
  h->have_step = true;
  return CMT_OK;
}

}  // namespace

// ================================================================================================
extern "C" {

int cmt_query_sizes(const cmt_config* cfg, size_t* param_bytes, size_t* grad_bytes, size_t* workspace_bytes) {
  if (!config_ok(cfg, nullptr)) return CMT_EINVAL;
  cmt_handle tmp;
  tmp.cfg = *cfg; tmp.prec = cfg->precision; tmp.esz = cfg->precision ? 2 : 4;
  tmp.Bpm = round_up(cfg->max_batch, 16);
  build_table(tmp.cfg, tmp.table, tmp.nparams);
  const size_t ws = layout(&tmp, nullptr);
  if (param_bytes) *param_bytes = tmp.nparams * 4;
  if (grad_bytes) *grad_bytes = tmp.nparams * 4;
  if (workspace_bytes) *workspace_bytes = ws;
  return CMT_OK;
}

int cmt_create(const cmt_config* cfg, void* params_dev, void* grads_dev, void* workspace_dev, void* hip_stream,
               cmt_handle** out) {
  if (!out) return CMT_EINVAL;
  *out = nullptr;
  std::string why;
  if (!config_ok(cfg, &why)) return CMT_EINVAL;
  if (!params_dev || !grads_dev || !workspace_dev) return CMT_EINVAL;
  if (((uintptr_t)params_dev | (uintptr_t)grads_dev | (uintptr_t)workspace_dev) & 255) return CMT_EINVAL;
  cmt_handle* h = new cmt_handle();
  h->cfg = *cfg; h->prec = cfg->precision; h->esz = cfg->precision ? 2 : 4;
  h->st = (hipStream_t)hip_stream;
  h->params = (float*)params_dev; h->grads = (float*)grads_dev; h->ws = (char*)workspace_dev;
  h->Bpm = round_up(cfg->max_batch, 16);
  {
    // k blocks of the encoder's k-split backward step GEMMs (up to L - 1 instances per launch): 2 (medium 9.72 ms
    // per step against 9.75 with 4, 9.86 with 8 and 9.96 with 1; large 24.59 / 24.69 / 24.71 / 24.74): fewer planes
    // for the consumer to sum weigh more than the extra workgroups, now that the operands stream fragment-major.
    // The decoder's k-split form launches one instance at a time and keeps as many blocks as fill the chip.
    const char* k1 = getenv("CMT_KB_BWD"); h->kb_bwd = k1 ? atoi(k1) : 2;
    const char* k1d = getenv("CMT_KB_BWD_DEC"); h->kb_bwd_dec = k1d ? atoi(k1d) : 0;
    const char* k2 = getenv("CMT_KB_WC"); h->kb_wc = k2 ? atoi(k2) : 2;
    const char* ks1 = getenv("CMT_SIDE_WGS"); h->side_wgs = ks1 ? atoi(ks1) : -1;
    const char* ks2 = getenv("CMT_SIDE_WGS_WO"); h->side_wgs_wo = ks2 ? atoi(ks2) : -1;
    const char* kw = getenv("CMT_WC_WHOLE_K"); h->wc_whole_k = kw ? atoi(kw) : 1;
    const char* k3 = getenv("CMT_SIDE_STREAM"); h->use_side = k3 ? atoi(k3) : 1;
    const char* k3p = getenv("CMT_ATT_PROJ"); h->att_proj = k3p ? atoi(k3p) : 1;
    const char* k4 = getenv("CMT_PHASE_TIMING"); h->phase_timing = k4 ? atoi(k4) : 0;
    const char* k5 = getenv("CMT_BWD_FUSED"); h->bwd_fused = k5 ? atoi(k5) : 5; h->bwd_fused_auto = k5 == nullptr;
  }
  build_table(h->cfg, h->table, h->nparams);
  h->ws_bytes = layout(h, h->ws);
  bind_params(h);
  hipError_t e = hipHostMalloc((void**)&h->h_loss, 256, hipHostMallocDefault);
  if (e != hipSuccess) { cmt_destroy(h); return CMT_EHIP; }
  // second stream at the default priority, and a pool of events for the hand-offs between the two
  if (hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking) != hipSuccess) { cmt_destroy(h); return CMT_EHIP; }
  h->ev.assign(512, nullptr);
  for (auto& ev : h->ev)
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { cmt_destroy(h); return CMT_EHIP; }
  h->h_flags = (int*)(h->h_loss + 8);
  h->h_loss[0] = 0.f; h->h_loss[1] = 0.f; *h->h_flags = 0;
  launch_fill_f32((float*)h->flags, 1, 0.f, h->st);  // the workspace may hold anything
  *out = h;
  return CMT_OK;
}

void cmt_destroy(cmt_handle* h) {
  if (!h) return;
  if (h->h_loss) (void)hipHostFree(h->h_loss);
  if (h->side) (void)hipStreamSynchronize(h->side);
  for (auto ev : h->ev) if (ev) (void)hipEventDestroy(ev);
  for (auto ev : h->phase_ev) if (ev) (void)hipEventDestroy(ev);
  if (h->side) (void)hipStreamDestroy(h->side);
  delete h;
}

int cmt_param_count(const cmt_handle* h) { return h ? (int)h->table.size() : CMT_EINVAL; }

int cmt_param_info(const cmt_handle* h, int idx, const char** name, int64_t* rows, int64_t* cols, size_t* offset_elems) {
  if (!h || idx < 0 || idx >= (int)h->table.size()) return CMT_EINVAL;
  const ParamInfo& p = h->table[idx];
  if (name) *name = p.name.c_str();
  if (rows) *rows = p.rows;
  if (cols) *cols = p.cols;
  if (offset_elems) *offset_elems = p.off;
  return CMT_OK;
}

int cmt_init_params(cmt_handle* h, uint64_t seed, float scale) {
  if (!h) return CMT_EINVAL;
  launch_init_uniform(h->params, h->nparams, seed, scale, h->st);
  refresh_params(h);
  hipError_t e = hipStreamSynchronize(h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_init_params");
  return CMT_OK;
}

int cmt_set_params(cmt_handle* h, const float* host_src) {
  if (!h || !host_src) return fail(h, CMT_EINVAL, "null pointer");
  hipError_t e = hipMemcpyAsync(h->params, host_src, h->nparams * 4, hipMemcpyHostToDevice, h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_set_params copy");
  refresh_params(h);
  e = hipStreamSynchronize(h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_set_params");
  return CMT_OK;
}

int cmt_get_params(cmt_handle* h, float* host_dst) {
  if (!h || !host_dst) return fail(h, CMT_EINVAL, "null pointer");
  hipError_t e = hipMemcpyAsync(host_dst, h->params, h->nparams * 4, hipMemcpyDeviceToHost, h->st);
  if (e == hipSuccess) e = hipStreamSynchronize(h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_get_params");
  return CMT_OK;
}

int cmt_get_grads(cmt_handle* h, float* host_dst) {
  if (!h || !host_dst) return fail(h, CMT_EINVAL, "null pointer");
  hipError_t e = hipMemcpyAsync(host_dst, h->grads, h->nparams * 4, hipMemcpyDeviceToHost, h->st);
  if (e == hipSuccess) e = hipStreamSynchronize(h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_get_grads");
  return CMT_OK;
}

int cmt_train_step_async(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev,
                         const int32_t* tgt_ids_dev, const int32_t* tgt_len_dev, int32_t B, int32_t S, int32_t T) {
  if (!h) return CMT_EINVAL;
  return enqueue_step(h, src_ids_dev, src_len_dev, tgt_ids_dev, tgt_len_dev, B, S, T, false);
}

int cmt_eval_loss(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, const int32_t* tgt_ids_dev,
                  const int32_t* tgt_len_dev, int32_t B, int32_t S, int32_t T, float* loss_host, float* n_tok_host) {
  if (!h) return CMT_EINVAL;
  const float keep_p = h->drop_p, keep_eps = h->ls_eps;
  h->drop_p = 0.f; h->ls_eps = 0.f;                 // evaluation: no masks, plain cross-entropy
  int rc = enqueue_step(h, src_ids_dev, src_len_dev, tgt_ids_dev, tgt_len_dev, B, S, T, true);
  h->drop_p = keep_p; h->ls_eps = keep_eps;
  if (rc != CMT_OK) return rc;
  rc = cmt_fetch_loss(h, loss_host);
  if (n_tok_host) *n_tok_host = h->h_loss[1];
  return rc;
}

// ---- evaluation without a caller-provided workspace -------------------------------------------------
// All intermediates of cmt_eval_loss_static live in this array instead of the handle's workspace.  In
// host code the array's name is only a stand-in: the device address comes from hipGetSymbolAddress,
// once per device (every GPU holds its own copy), and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[CMT_STATIC_SCRATCH_BYTES];
namespace {
constexpr int STATIC_MAX_DEVICES = 64;
void* g_static_scratch[STATIC_MAX_DEVICES] = {};
// device address of `scratch` on the current device (looked up at the first call on that device)
int static_scratch_ptr(cmt_handle* h, char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(h, e, "hipGetDevice");
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(h, CMT_EINVAL, "device ordinal beyond the static scratch table");
  if (!g_static_scratch[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(h, e, "hipGetSymbolAddress(scratch)");
    g_static_scratch[dev] = p;
  }
  *out = (char*)g_static_scratch[dev];
  return CMT_OK;
}
}  // namespace

int cmt_eval_loss_static(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, const int32_t* tgt_ids_dev,
                         const int32_t* tgt_len_dev, int32_t B, int32_t S, int32_t T, float* loss_host, float* n_tok_host) {
  if (!h) return CMT_EINVAL;
  const cmt_config& c = h->cfg;
  if (B < 1 || B > c.max_batch || S < 1 || S > c.max_src_len || T < 1 || T > c.max_tgt_len)
    return fail(h, CMT_EINVAL, "B, S or T outside [1, configured maximum]");
  // a view of the handle whose workspace is the static array, laid out for exactly this call's shape
  cmt_handle v = *h;
  v.cfg.max_batch = B; v.cfg.max_src_len = S; v.cfg.max_tgt_len = T;
  v.Bpm = round_up(B, 16);
  v.phase_timing = 0; v.phase_ev.clear(); v.phase_name.clear();
  const size_t need = layout(&v, nullptr);
  if (need > (size_t)CMT_STATIC_SCRATCH_BYTES) {
    char msg[160];
    snprintf(msg, sizeof msg, "this shape needs %zu bytes of scratch, the static buffer holds %zu", need,
             (size_t)CMT_STATIC_SCRATCH_BYTES);
    return fail(h, CMT_EINVAL, msg);
  }
  char* base = nullptr;
  int rc = static_scratch_ptr(h, &base);
  if (rc != CMT_OK) return rc;
  v.ws = base;
  v.ws_bytes = layout(&v, base);
  bind_params(&v);
  // the array keeps the last call's contents (perhaps of another shape): start from zeros
  launch_fill_f32((float*)base, (need + 3) / 4, 0.f, v.st);
  refresh_params(&v);                                // working copies of the parameters (casts, transposes) in the array
  v.drop_p = 0.f; v.ls_eps = 0.f;                    // evaluation: no masks, plain cross-entropy
  rc = enqueue_step(&v, src_ids_dev, src_len_dev, tgt_ids_dev, tgt_len_dev, B, S, T, true);
  if (rc == CMT_OK) rc = cmt_fetch_loss(&v, loss_host);
  if (rc != CMT_OK) { h->err = v.err; return rc; }
  if (n_tok_host) *n_tok_host = v.h_loss[1];
  h->ev_next = v.ev_next;
  return CMT_OK;
}

int cmt_fetch_loss(cmt_handle* h, float* loss_host) {
  if (!h) return CMT_EINVAL;
  if (!h->have_step) return fail(h, CMT_EINVAL, "no step has been run");
  hipError_t e = hipStreamSynchronize(h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_fetch_loss");
  if (h->phase_timing && h->phase_n > 1) {          // phases of the last step, as the caller's stream saw them
    float total = 0.f;
    for (size_t i = 0; i + 1 < h->phase_n; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, h->phase_ev[i], h->phase_ev[i + 1]) != hipSuccess) break;
      fprintf(stderr, "[cytonmt_hip] %-40s %8.3f ms   (enqueued in %6.3f ms)\n", h->phase_name[i], ms,
              h->phase_host[i + 1] - h->phase_host[i]);
      total += ms;
    }
    fprintf(stderr, "[cytonmt_hip] %-40s %8.3f ms\n", "step", total);
  }
  const int flags = *h->h_flags;
  if (loss_host) *loss_host = h->h_loss[0];
  if (flags) {                                       // reported once: clear the device word for the steps to come
    *h->h_flags = 0;
    launch_fill_f32((float*)h->flags, 1, 0.f, h->st);
  }
  if (flags & 3) return fail(h, CMT_ERANGE, (flags & 1) ? "a token id is outside its vocabulary" : "a length is outside [1, padded length]");
  if (flags & 4) return fail(h, CMT_ENONFINITE, "the loss is not finite");
  return CMT_OK;
}

int cmt_train_step(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, const int32_t* tgt_ids_dev,
                   const int32_t* tgt_len_dev, int32_t B, int32_t S, int32_t T, float* loss_host) {
  const int rc = cmt_train_step_async(h, src_ids_dev, src_len_dev, tgt_ids_dev, tgt_len_dev, B, S, T);
  if (rc != CMT_OK) return rc;
  return cmt_fetch_loss(h, loss_host);
}

int cmt_greedy_decode(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, int32_t B, int32_t S,
                      int32_t max_len, int32_t eos_id, int32_t* out_ids_dev, int32_t* out_len_dev) {
  if (!h) return CMT_EINVAL;
  const cmt_config& c = h->cfg;
  if (!src_ids_dev || !src_len_dev || !out_ids_dev || !out_len_dev) return fail(h, CMT_EINVAL, "null pointer");
  if (B < 1 || B > c.max_batch || S < 1 || S > c.max_src_len || max_len < 1 || max_len > c.max_tgt_len)
    return fail(h, CMT_EINVAL, "B, S or max_len outside [1, configured maximum]");
  if (eos_id < 0 || eos_id >= c.tgt_vocab) return fail(h, CMT_EINVAL, "eos_id outside the target vocabulary");
  const int p = h->prec, E = c.emb_dim, H = c.hidden, L = c.layers, V = c.tgt_vocab;
  const int Bp = round_up(B, 16);
  const size_t esz = h->esz;
  hipStream_t st = h->st;
  h->B = B; h->Bp = Bp; h->S = S; h->T = max_len;
  h->have_step = false;                              // the training step's intermediates are overwritten
  h->phase_n = 0;
  const int PH = h->PH;
  const size_t BP = (size_t)Bp * PH, BH = (size_t)Bp * H;
  const float keep_p = h->drop_p;
  h->drop_p = 0.f;                                   // inference: no dropout
  launch_fill_f32((float*)h->flags, 1, 0.f, st);
  launch_gather(p, h->Pw(h->off_Esrc), c.src_vocab, E, src_ids_dev, src_len_dev, B, Bp, S, 0, 0, h->Xs, h->mask_s, h->tok_s,
                nullptr, h->len_s, h->flags, st);
  const char* Hs; int ldHs;
  enqueue_encoder(h, S, &Hs, &ldHs);
  const bool proj = h->att_proj && Bp < 256;
  if (proj) launch_gemm_nt(p, Hs, ldHs, h->Pw(h->off_Wc), 2 * H, S * Bp, H, H, nullptr, h->PmatT, H, nullptr, 0, st);
  launch_dec_init(B, Bp, max_len, c.bos_id, c.pad_id, h->dec_tok, h->dec_done, out_ids_dev, out_len_dev, h->dec_mask, st);
  launch_fill_T(p, h->xcat, (size_t)Bp * h->ldxcat, st);              // H_o^{<-1>} = 0
  const bool fm0 = h->xcatF && h->dec[0].fm;                          // bottom layer on fragment-major operands
  if (fm0) launch_fill_T(p, h->xcatF, (size_t)Bp * (E + H), st);
  // the first step's input embedding; every later one is written by the arg-max kernel of the step before
  launch_dec_embed(p, h->Pw(h->off_Etgt), E, h->dec_tok, B, Bp, h->xcat, h->ldxcat, st, fm0 ? h->xcatF : nullptr, (E + H) >> 5);
  for (int j = 0; j < max_len; ++j) {
    for (int l = 0; l < L; ++l) {
      LD& e = h->dec[l];
      LstmFwdDir d;
      if (l == 0) { d.x = h->xcat; d.ldx = h->ldxcat; d.Kx = E + H; d.wx_off = 0; d.wh_off = E + H; d.ldw = E + 2 * H; }
      else { d.x = h->dec[l - 1].Hst + (j + 1) * BP * esz; d.ldx = e.ph; d.Kx = H; d.wx_off = 0; d.wh_off = H; d.ldw = 2 * H; }
      d.gx = nullptr; d.ldgx = 0; d.bias = h->params + e.b_off;
      d.hprev = e.Hst + j * BP * esz; d.ldh = e.ph; d.W = e.W;
      d.cprev = e.Cst + j * BH; d.mask = h->dec_mask;
      d.hnext = e.Hst + (j + 1) * BP * esz; d.ldhn = e.ph; d.cnext = e.Cst + (j + 1) * BH;
      d.gsave = e.Gs + (size_t)j * Bp * 4 * H; d.ycat = nullptr; d.ldy = 0;
      if (e.fm) {
        d.hnext_fm = e.HstF + (j + 1) * BH * esz;
        if (l > 0 && h->dec[l - 1].fm) {
          d.W_fm = e.Wfm; d.x_fm = h->dec[l - 1].HstF + (j + 1) * BH * esz; d.hprev_fm = e.HstF + j * BH * esz;
        } else if (l == 0 && fm0) {
          d.W_fm = h->Wdec0F; d.x_fm = h->xcatF; d.hprev_fm = e.HstF + j * BH * esz;
        }
      }
      launch_lstm_fwd(p, &d, 1, Bp, H, st);
    }
    const char* Ht = h->dec[L - 1].Hst + (j + 1) * BP * esz;
    StepGemm g{};                                   // H_o = tanh(W_c [C_s; H_t]) straight into the next step's input
    g.a0 = h->Cs + j * BP * esz; g.lda0 = PH; g.K0 = H; g.w0_off = 0;
    g.a1 = Ht; g.lda1 = PH; g.K1 = H; g.w1_off = H;
    g.W = h->Pw(h->off_Wc); g.ldw = 2 * H; g.N = H; g.mode = 0;
    g.outT = h->xcat + (size_t)E * esz; g.ldo = h->ldxcat;
    g.out = h->wcp; g.ldout = H; g.plane_stride = BH;
    if (h->HoFeedF && h->dec[L - 1].fm) {
      g.W_fm = h->WcF; g.a0_fm = h->CsF + j * BH * esz; g.a1_fm = h->dec[L - 1].HstF + (j + 1) * BH * esz;
      g.outF = h->HoFeedF;                          // H_o of this step, for the logits
      if (fm0) { g.outF2 = h->xcatF; g.outF2_nsteps = (E + H) >> 5; g.outF2_k0 = E; }   // and for the next step's bottom layer
    }
    if (proj) {                                     // on the projected source rows, as in the training step
      AttOut o{};
      o.outT = g.outT; o.ldo = g.ldo; o.outF = g.outF; o.outF2 = g.outF2; o.outF2_nsteps = g.outF2_nsteps; o.outF2_k0 = g.outF2_k0;
      g.mode = 3; g.skip0 = 1; g.a0_fm = g.a1_fm;
      launch_att_fwd_proj(p, h->Kmat, H, h->PmatT, H, Ht, PH, g, o, h->len_s, S, Bp, H, h->dots, h->att_a + (size_t)j * Bp * S, st);
    } else {
      launch_att_fwd(p, h->Kmat, H, Hs, ldHs, Ht, PH, h->len_s, S, Bp, H, h->dots, h->att_a + (size_t)j * Bp * S,
                     h->Cs + j * BP * esz, PH, st, h->CsF ? h->CsF + j * BH * esz : nullptr);
      launch_step_gemm(p, g, Bp, st);
    }
    StepGemm z{};                                   // logits (without the bias) = H_o W_o^T
    z.a0 = h->xcat + (size_t)E * esz; z.lda0 = h->ldxcat; z.K0 = H; z.w0_off = 0; z.K1 = 0;
    // ... of which only the largest per sentence is wanted: every workgroup of the product keeps the best of its 64
    // vocabulary entries (bias included), and the arg-max kernel picks among those
    const int nblk = (V + 63) / 64;
    float* part_v = h->logits; int32_t* part_i = (int32_t*)(h->logits + (size_t)nblk * Bp);
    z.W = h->Pw(h->off_Wo); z.ldw = H; z.N = V; z.mode = 2; z.max_kb = 1;
    if (g.outF && h->WoF) { z.W_fm = h->WoF; z.a0_fm = h->HoFeedF; }
    z.out = part_v; z.best_idx = part_i; z.bias = h->params + h->off_Bo; z.ldout = V; z.plane_stride = (size_t)Bp * V;
    launch_step_gemm(p, z, Bp, st);
    launch_dec_argmax(part_v, Bp, nullptr, nblk, B, j, max_len, eos_id, h->dec_tok, h->dec_done, out_ids_dev,
                      out_len_dev, st, p, h->Pw(h->off_Etgt), E, h->xcat, h->ldxcat, fm0 ? h->xcatF : nullptr, (E + H) >> 5, part_i);
  }
  h->drop_p = keep_p;
  (void)hipMemcpyAsync(h->h_flags, h->flags, sizeof(int), hipMemcpyDeviceToHost, st);
  hipError_t e = hipStreamSynchronize(st);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "cmt_greedy_decode");
  const int flags = *h->h_flags;
  if (flags & 3) return fail(h, CMT_ERANGE, (flags & 1) ? "a token id is outside its vocabulary" : "a length is outside [1, padded length]");
  return CMT_OK;
}

int cmt_beam_decode(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, int32_t B, int32_t S,
                    int32_t max_len, int32_t beam, float length_penalty, int32_t eos_id, int32_t* out_ids_dev,
                    int32_t* out_len_dev, float* out_score_dev) {
  if (!h) return CMT_EINVAL;
  const cmt_config& c = h->cfg;
  if (!src_ids_dev || !src_len_dev || !out_ids_dev || !out_len_dev || !out_score_dev) return fail(h, CMT_EINVAL, "null pointer");
  if (B < 1 || S < 1 || S > c.max_src_len || max_len < 1 || max_len > c.max_tgt_len)
    return fail(h, CMT_EINVAL, "B, S or max_len outside [1, configured maximum]");
  if (beam < 1 || beam > 16) return fail(h, CMT_EINVAL, "beam must be in [1, 16]");
  if ((long long)B * beam > c.max_batch) return fail(h, CMT_EINVAL, "B * beam exceeds max_batch (one decoder row per hypothesis)");
  if (c.max_tgt_len < 2) return fail(h, CMT_EINVAL, "beam search needs max_tgt_len >= 2 (state double buffer)");
  if (!(length_penalty >= 0.f) || !isfinite(length_penalty)) return fail(h, CMT_EINVAL, "length_penalty must be finite and >= 0");
  if (eos_id < 0 || eos_id >= c.tgt_vocab) return fail(h, CMT_EINVAL, "eos_id outside the target vocabulary");
  const int p = h->prec, E = c.emb_dim, H = c.hidden, L = c.layers, V = c.tgt_vocab, K = beam;
  const int BpE = round_up(B, 16);                   // encoder rows
  const int R = B * K, Rp = round_up(R, 16);         // decoder rows
  const size_t esz = h->esz;
  hipStream_t st = h->st;
  h->B = B; h->Bp = BpE; h->S = S; h->T = max_len;
  h->have_step = false;
  h->phase_n = 0;
  const int PH = h->PH;
  const float keep_p = h->drop_p;
  h->drop_p = 0.f;                                   // inference: no dropout
  launch_fill_f32((float*)h->flags, 1, 0.f, st);
  launch_gather(p, h->Pw(h->off_Esrc), c.src_vocab, E, src_ids_dev, src_len_dev, B, BpE, S, 0, 0, h->Xs, h->mask_s, h->tok_s,
                nullptr, h->len_s, h->flags, st);
  const char* Hs; int ldHs;
  enqueue_encoder(h, S, &Hs, &ldHs);                 // also leaves the decoder's initial states in slot 0 (BpE rows)
  h->drop_p = keep_p;
  // one decoder row per hypothesis: encoder outputs, keys, lengths and initial states repeated K times
  BeamState& bs = h->beam;
  bs.hist_ld = Rp;
  launch_beam_init(bs, B, Rp, K, c.bos_id, h->len_s, h->len_exp, st);
  // (below 256 rows the attention runs on the projected source rows, as in the training step: those are expanded
  // in the place of the source states)
  const bool proj = h->att_proj && Rp < 256;
  if (proj) {
    launch_gemm_nt(p, Hs, ldHs, h->Pw(h->off_Wc), 2 * H, S * BpE, H, H, nullptr, h->PmatT, H, nullptr, 0, st);
    launch_beam_expand((int)esz, h->PmatT, H, BpE, h->Hs_exp, H, S, R, Rp, K, H, st);
  } else {
    launch_beam_expand((int)esz, Hs, ldHs, BpE, h->Hs_exp, H, S, R, Rp, K, H, st);
  }
  launch_beam_expand((int)esz, h->Kmat, H, BpE, h->K_exp, H, S, R, Rp, K, H, st);
  const size_t slotT = (size_t)Rp * PH * esz, slotC = (size_t)Rp * H * 4;   // state slots of Rp rows: 1 = read, 2 = written
  const size_t slotF = (size_t)Rp * H * esz;                                // the same slots of the fragment-major copies
  for (int l = 0; l < L; ++l) {
    LD& e = h->dec[l];
    launch_beam_expand((int)esz, e.Hst, e.ph, BpE, e.Hst + slotT, e.ph, 1, R, Rp, K, H, st);
    launch_beam_expand(4, e.Cst, H, BpE, (char*)e.Cst + slotC, H, 1, R, Rp, K, H, st);
    if (e.fm) launch_fm_pack(e.Hst + slotT, e.ph, Rp, H, e.HstF + slotF, st);   // fragment-major copy of the expanded states
  }
  launch_fill_T(p, h->xcat, (size_t)Rp * h->ldxcat, st);               // H_o^{<-1>} = 0
  const bool fm0 = h->xcatF && h->dec[0].fm;                           // bottom layer on fragment-major operands
  if (fm0) launch_fill_T(p, h->xcatF, (size_t)Rp * (E + H), st);
  BeamReorder ro{};
  for (int l = 0; l < L; ++l) {
    LD& e = h->dec[l];
    ro.h_src[l] = e.Hst + 2 * slotT; ro.h_dst[l] = e.Hst + slotT;
    ro.c_src[l] = (const float*)((char*)e.Cst + 2 * slotC); ro.c_dst[l] = (float*)((char*)e.Cst + slotC);
    if (e.fm) ro.h_dst_fm[l] = e.HstF + slotF;
  }
  ro.ldh = PH;
  ro.ho_src = h->HoBuf; ro.ldho_src = PH; ro.ho_dst = h->xcat + (size_t)E * esz; ro.ldho_dst = h->ldxcat;
  if (fm0) { ro.ho_dst_fm = h->xcatF; ro.ho_fm_nsteps = (E + H) >> 5; ro.ho_fm_k0 = E; }
  for (int j = 0; j < max_len; ++j) {
    launch_dec_embed(p, h->Pw(h->off_Etgt), E, bs.tok, R, Rp, h->xcat, h->ldxcat, st, fm0 ? h->xcatF : nullptr, (E + H) >> 5);
    for (int l = 0; l < L; ++l) {
      LD& e = h->dec[l];
      LstmFwdDir d;
      if (l == 0) { d.x = h->xcat; d.ldx = h->ldxcat; d.Kx = E + H; d.wx_off = 0; d.wh_off = E + H; d.ldw = E + 2 * H; }
      else { d.x = h->dec[l - 1].Hst + 2 * slotT; d.ldx = PH; d.Kx = H; d.wx_off = 0; d.wh_off = H; d.ldw = 2 * H; }
      d.gx = nullptr; d.ldgx = 0; d.bias = h->params + e.b_off;
      d.hprev = e.Hst + slotT; d.ldh = e.ph; d.W = e.W;
      d.cprev = (const float*)((char*)e.Cst + slotC); d.mask = bs.mask;
      d.hnext = e.Hst + 2 * slotT; d.ldhn = e.ph; d.cnext = (float*)((char*)e.Cst + 2 * slotC);
      d.gsave = e.Gs; d.ycat = nullptr; d.ldy = 0;
      if (e.fm) {                                    // as in greedy decoding: the layers above the bottom one
        d.hnext_fm = e.HstF + 2 * slotF;
        if (l > 0 && h->dec[l - 1].fm) { d.W_fm = e.Wfm; d.x_fm = h->dec[l - 1].HstF + 2 * slotF; d.hprev_fm = e.HstF + slotF; }
        else if (l == 0 && fm0) { d.W_fm = h->Wdec0F; d.x_fm = h->xcatF; d.hprev_fm = e.HstF + slotF; }
      }
      launch_lstm_fwd(p, &d, 1, Rp, H, st);
    }
    const char* Ht = h->dec[L - 1].Hst + 2 * slotT;
    StepGemm g{};
    g.a0 = h->Cs; g.lda0 = PH; g.K0 = H; g.w0_off = 0;
    g.a1 = Ht; g.lda1 = PH; g.K1 = H; g.w1_off = H;
    g.W = h->Pw(h->off_Wc); g.ldw = 2 * H; g.N = H; g.mode = 0;
    g.outT = h->HoBuf; g.ldo = PH;
    g.out = h->wcp; g.ldout = H; g.plane_stride = (size_t)Rp * H;
    if (h->CsF && h->dec[L - 1].fm) { g.W_fm = h->WcF; g.a0_fm = h->CsF; g.a1_fm = h->dec[L - 1].HstF + 2 * slotF; }
    if (proj) {
      AttOut o{};
      o.outT = g.outT; o.ldo = g.ldo;
      g.mode = 3; g.skip0 = 1; g.a0_fm = g.a1_fm;
      launch_att_fwd_proj(p, h->K_exp, H, h->Hs_exp, H, Ht, PH, g, o, h->len_exp, S, Rp, H, h->dots, h->att_a, st);
    } else {
      launch_att_fwd(p, h->K_exp, H, h->Hs_exp, H, Ht, PH, h->len_exp, S, Rp, H, h->dots, h->att_a, h->Cs, PH, st, h->CsF);
      launch_step_gemm(p, g, Rp, st);
    }
    launch_gemm_nt(p, h->HoBuf, PH, h->Pw(h->off_Wo), H, Rp, V, H, h->logits, nullptr, V, h->params + h->off_Bo, 0, st);
    launch_beam_select(h->logits, V, bs, B, K, j, max_len, eos_id, length_penalty, st, p);
    launch_beam_reorder(p, ro, bs, R, H, L, st);
  }
  launch_beam_finish(bs, B, K, max_len, c.pad_id, out_ids_dev, out_len_dev, out_score_dev, st);
  (void)hipMemcpyAsync(h->h_flags, h->flags, sizeof(int), hipMemcpyDeviceToHost, st);
  hipError_t e = hipStreamSynchronize(st);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "cmt_beam_decode");
  const int flags = *h->h_flags;
  if (flags & 3) return fail(h, CMT_ERANGE, (flags & 1) ? "a token id is outside its vocabulary" : "a length is outside [1, padded length]");
  return CMT_OK;
}

int cmt_sgd_update(cmt_handle* h, float lr) {
  if (!h) return CMT_EINVAL;
  if (!isfinite(lr)) return fail(h, CMT_EINVAL, "learning rate is not finite");
  launch_sgd(h->params, h->grads, h->nparams, lr, h->flags, h->prec ? h->Pc : nullptr, h->st);
  refresh_params(h, false);                        // the update wrote the bf16 copy itself: only the transposes are left
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "cmt_sgd_update");
  return CMT_OK;
}

int cmt_set_regularization(cmt_handle* h, float dropout, float label_smoothing, uint64_t dropout_seed) {
  if (!h) return CMT_EINVAL;
  if (!(dropout >= 0.f) || !(dropout < 1.f)) return fail(h, CMT_EINVAL, "dropout must be in [0, 1)");
  if (!(label_smoothing >= 0.f) || !(label_smoothing < 1.f)) return fail(h, CMT_EINVAL, "label_smoothing must be in [0, 1)");
  h->drop_p = dropout;
  h->drop_thresh = (unsigned)floor((double)dropout * 16777216.0);
  h->drop_scale = (float)(1.0 / (1.0 - (double)dropout));
  h->drop_seed = dropout_seed;
  h->ls_eps = label_smoothing;
  return CMT_OK;
}

int cmt_time_kernel(cmt_handle* h, const char* name, int iters, float* us_per_launch, double* algo_work) {
  if (!h || !name || iters < 1 || !us_per_launch || !algo_work) return fail(h, CMT_EINVAL, "bad argument");
  if (!h->have_step) return fail(h, CMT_EINVAL, "no step has been run");
  const cmt_config& c = h->cfg;
  const int p = h->prec, H = c.hidden, L = c.layers, E = c.emb_dim, V = c.tgt_vocab, Bp = h->Bp, T = h->T, S = h->S;
  const int PH = h->PH, Mt = T * Bp;
  const size_t BP = (size_t)Bp * PH, BH = (size_t)Bp * H;
  const double esz = (double)h->esz;
  const size_t es = h->esz;
  hipStream_t st = h->st;
  const std::string s(name);
  const int j = T / 2;                                  // the middle target position
  std::function<void(int)> launch;
  const int* probe_flag = nullptr;                      // set by a probe whose bounded wait may give up
  if (s == "lstm_fwd_dec") {
    // decoder LSTM forward step, cycling over the layers like the real loop (weights not L2-resident)
    const int K = 2 * H;                                // per-step contraction (layer 0: [feed; h], others: [x; h])
    *algo_work = 4.0 * H * K * esz                      // weights, read once
               + (double)Bp * K * esz                   // [x; h_prev]
               + (double)4 * H * 4                      // bias (the layers timed here have no pre-batched input part)
               + (double)Bp * H * 4                     // c_prev
               + (double)Bp * H * (esz + 4)             // h, c out
               + (double)Bp * 4 * H * 4;                // gate activations kept for backward
    launch = [=](int i) { dec_lstm_fwd(h, L > 1 ? 1 + i % (L - 1) : 0, j); };
  } else if (s == "step2d_bwd_dec") {
    // [dx; dh_prev] = dgates [W_x; W_h] of a decoder layer, written as planes
    const int kb = step_kblocks(p, 2 * H, 4 * H, Bp, h->kb_bwd_dec);
    *algo_work = 4.0 * H * 2 * H * esz + (double)Bp * 4 * H * esz + (double)kb * Bp * 2 * H * 4;
    launch = [=](int i) {
      LD& e = h->dec[L > 1 ? 1 + i % (L - 1) : 0];
      StepGemm g{};
      g.a0 = e.dG + (size_t)j * Bp * e.pg * es; g.lda0 = e.pg; g.K0 = 4 * H; g.w0_off = 0; g.K1 = 0;
      g.W = e.Wt + (size_t)(&e == &h->dec[0] ? E : 0) * 4 * H * es; g.ldw = 4 * H;
      g.N = 2 * H; g.mode = 1; g.max_kb = h->kb_bwd_dec;
      g.out = e.bwdp; g.ldout = 2 * H; g.plane_stride = (size_t)Bp * 2 * H;
      if (e.fmb) { g.W_fm = e.WtF; g.w_tile0 = (&e == &h->dec[0] ? E : 0) / 16; g.a0_fm = e.dGF + (size_t)j * Bp * 4 * H * es; }
      launch_step_gemm(p, g, Bp, st);
    };
  } else if (s == "step_bwd_fused_dec") {
    // the same product with the whole contraction inside the workgroup and the cell backward of the layer below
    // in the epilogue (the form the decoder's backward loop runs): weights and dgates read once, dh_prev stored,
    // and the pointwise operands of the fused cell backward (gates, c, dc, dh in and out, dgates out)
    *algo_work = 4.0 * H * 2 * H * esz + (double)Bp * 4 * H * esz + (double)Bp * H * 4
               + (double)Bp * H * (4 * 4 + 2 * 4 + 2 * 4 + 2 * 4 + 4) + (double)Bp * 4 * H * esz;
    launch = [=](int i) {
      const StepBwd g = dec_bwd_gemm(h, L > 1 ? 1 + i % (L - 1) : 0, j);
      launch_step_bwd_fused(p, &g, 1, Bp, st);
    };
  } else if (s == "att_fwd") {
    // attention forward of one decoder step as the step launches it.  On the projected rows: scores (with the sums
    // W_c2 H_t in the same launch), softmax, mix and tanh -> H_o: the keys and the projected rows of every sentence
    // once and the H_t half of W_c.  Else scores + softmax + context: the keys and H_s of every sentence once.
    const bool proj = h->att_proj && Bp < 256;
    *algo_work = 2.0 * Bp * S * H * esz + (proj ? (double)H * H * esz : 0.0);
    const char* Hs = L > 1 ? h->enc[L].Hst + BP * es : h->Y0;
    const int ldHs = L > 1 ? PH : H;
    launch = [=](int) {
      if (proj) dec_att_fwd_proj(h, j, S, h->dots);
      else launch_att_fwd(p, h->Kmat, H, Hs, ldHs, h->dec[L - 1].Hst + (j + 1) * BP * es, PH, h->len_s, S, Bp, H, h->dots,
                          h->att_a + (size_t)j * Bp * S, h->Cs + j * BP * es, PH, st);
    };
  } else if (s == "att_bwd") {
    // attention backward of one decoder step as the step launches it (score gradients, the gradient sent to the
    // top layer's output, that layer's cell backward in the same launch).  On the projected rows the launch of
    // dpre W_c is part of it: the fp32 projected rows and the keys of every sentence once, and W_c.  Else H_s and the
    // keys of every sentence once.
    const bool fused = (h->bwd_fused & 1) && Bp <= 128;
    const bool proj = (h->att_proj & 1) && Bp < 256 && fused && h->wc_whole_k;
    *algo_work = proj ? (double)Bp * S * H * (4 + esz) + 2.0 * H * H * esz : 2.0 * Bp * S * H * esz;
    const char* Hs = L > 1 ? h->enc[L].Hst + BP * es : h->Y0;
    const int ldHs = L > 1 ? PH : H;
    // (the planes the step's dpre W_c wrote: one in the fused loop's whole-k form)
    const int kbw = (h->wc_whole_k && fused) ? 1 : step_kblocks(p, 2 * H, H, Bp, h->kb_wc);
    const size_t pstr = (size_t)Bp * 2 * H;
    launch = [=](int) {
      if (proj) { dec_att_bwd_proj(h, j, S, false); return; }
      LstmBwdPoint top = dec_cell(h, L - 1, j);
      top.dhrec = Planes{h->dec[L - 1].bwdp, H, 1, 0};
      launch_att_bwd(p, h->Kmat, H, Hs, ldHs, Planes{h->wcp, 2 * H, kbw, pstr}, h->dCs + j * BH, h->att_a + (size_t)j * Bp * S,
                     h->len_s, S, Bp, H, h->dots, h->att_ds + (size_t)j * Bp * S, h->dHt, st, &top);
    };
  } else if (s == "gemm_gx") {
    // time-batched input-side GEMM of the decoder's bottom layer: [T Bp, E] x [E, 4H]  (flops)
    *algo_work = 2.0 * Mt * 4 * H * E;
    launch = [=](int) {
      LD& d0 = h->dec[0];
      launch_gemm_nt(p, h->Xt, E, d0.W, E + 2 * H, Mt, 4 * H, E, d0.Gx, nullptr, 4 * H, h->params + d0.b_off, 0, st);
    };
  } else if (s == "gemm_dw") {
    // the decoder's weight gradients as the step launches them: W_c (two segments) and every layer's segments,
    // dG^T [4H, T Bp] x X^T [width, T Bp]^T each, one grouped launch  (flops)
    std::vector<GemmProb> probs;
    probs.push_back(GemmProb{h->dPreT, h->CsT, h->grads + h->off_Wc, Mt, Mt, 2 * H, H, H, Mt, 0});
    probs.push_back(GemmProb{h->dPreT, h->dec[L - 1].HstT + (size_t)Bp * es, h->grads + h->off_Wc + H, Mt, (T + 1) * Bp, 2 * H, H, H, Mt, 0});
    for (int l = 0; l < L; ++l) {
      LD& e = h->dec[l];
      float* dW = h->grads + e.w_off;
      if (l == 0) {
        probs.push_back(GemmProb{e.dGT, h->XtT, dW, Mt, Mt, e.Kin + H, 4 * H, E, Mt, 0});
        probs.push_back(GemmProb{e.dGT, h->HoBufT, dW + E, Mt, Mt + Bp, e.Kin + H, 4 * H, H, Mt, 0});
        probs.push_back(GemmProb{e.dGT, e.HstT, dW + E + H, Mt, (T + 1) * Bp, e.Kin + H, 4 * H, H, Mt, 0});
      } else {
        if (h->drop_p > 0.f) probs.push_back(GemmProb{e.dGT, h->dec[l - 1].YdT, dW, Mt, Mt, e.Kin + H, 4 * H, H, Mt, 0});
        else probs.push_back(GemmProb{e.dGT, h->dec[l - 1].HstT + (size_t)Bp * es, dW, Mt, (T + 1) * Bp, e.Kin + H, 4 * H, H, Mt, 0});
        probs.push_back(GemmProb{e.dGT, e.HstT, dW + H, Mt, (T + 1) * Bp, e.Kin + H, 4 * H, H, Mt, 0});
      }
    }
    double fl = 0;
    for (const GemmProb& q : probs) fl += 2.0 * q.M * q.N * q.K;
    *algo_work = fl;
    launch = [=](int) { launch_gemm_nt_group(p, probs.data(), (int)probs.size(), st, h->gsplit2, h->gsplit2_floats); };
  } else if (s == "ce_fwd") {
    // vocabulary projection of one slab of rows with the partial log-sum-exp statistics  (flops)
    int nslab;
    const int rows = ce_slab_plan(h, Mt, &nslab);
    const int Mc = nslab == 1 ? Mt : rows;              // the first slab
    *algo_work = 2.0 * Mc * (double)V * H;
    const char* Ho = (h->drop_p > 0.f ? h->HoDrop : h->HoBuf) + BP * es;
    launch = [=](int) {
      launch_ce_fwd(p, Ho, PH, h->Pw(h->off_Wo), h->params + h->off_Bo, h->labels, Mc, V, H, h->dzTs, h->ce_pitch, h->pmax,
                    h->psum, nullptr, h->zy, st);
    };
  } else if (s == "grid_barrier" || s == "grid_barrier_nofence") {
    // 100 chip-wide barriers between 256 resident workgroups (bounded polling); work = the number of barriers
    const int rounds = 100, fences = s == "grid_barrier" ? 1 : 0;
    unsigned* counter = (unsigned*)h->gsplit;
    int* gave_up = (int*)h->gsplit + 64;
    *algo_work = rounds;
    launch = [=](int) {
      launch_fill_f32(h->gsplit, 128, 0.f, st);
      launch_grid_barrier_probe(counter, gave_up, 256, rounds, fences, 1 << 16, st);
    };
    probe_flag = gave_up;
  } else if (s == "mfma_rate") {
    // matrix cores alone: up to 4096 workgroups x 4 wavefronts x 2048 x 4 bf16 32x32x16 MFMAs on registers  (flops)
    const int it = 2048;
    const int blocks = (int)std::min<size_t>(4096, h->gsplit_floats / 256);   // one float per lane lands in the split-k scratch
    if (blocks < 1) return fail(h, CMT_EINVAL, "workspace too small for the probe");
    *algo_work = (double)blocks * 4 * it * 4.0 * (2.0 * 32 * 32 * 16);
    launch = [=](int) { (void)launch_mfma_rate(h->gsplit, blocks, it, st); };
  } else {
    return fail(h, CMT_EINVAL, "unknown kernel name");
  }
  (void)BH;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return fail(h, CMT_EHIP, "event create");
  for (int i = 0; i < 4; ++i) launch(i);
  (void)hipEventRecord(e0, st);
  for (int i = 0; i < iters; ++i) launch(i);
  (void)hipEventRecord(e1, st);
  hipError_t e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_time_kernel");
  *us_per_launch = ms * 1e3f / iters;
  if (probe_flag) {
    int gave = 0;
    e = hipMemcpy(&gave, probe_flag, sizeof(int), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e, "cmt_time_kernel");
    if (gave) return fail(h, CMT_EHIP, "the barrier probe gave up waiting (its workgroups were not all resident)");
  }
  return CMT_OK;
}

int cmt_padded_batch(const cmt_handle* h) { return h ? h->Bp : CMT_EINVAL; }

int cmt_debug_fetch(cmt_handle* h, const char* name, float* host_dst, size_t bytes) {
  if (!h || !name || !host_dst) return fail(h, CMT_EINVAL, "null pointer");
  if (!h->have_step) return fail(h, CMT_EINVAL, "no step has been run");
  const int H = h->cfg.hidden, E = h->cfg.emb_dim, L = h->cfg.layers;
  const size_t Bp = h->Bp, S = h->S, T = h->T, BP = Bp * h->PH;
  // rows x cols elements with a source row pitch (elements); isT: stored in the operand type
  const void* src = nullptr; size_t rows = 0, cols = 0, pitch = 0; bool isT = false;
  const std::string s(name);
  if (s == "x_src") { src = h->Xs; rows = S * Bp; cols = pitch = E; isT = true; }
  else if (s == "x_tgt") { src = h->Xt; rows = T * Bp; cols = pitch = E; isT = true; }
  else if (s == "mask_src") { src = h->mask_s; rows = 1; cols = pitch = S * Bp; }
  else if (s == "mask_tgt") { src = h->mask_t; rows = 1; cols = pitch = T * Bp; }
  else if (s == "h_s") {
    rows = S * Bp; cols = H; isT = true;
    if (L == 1) { src = h->Y0; pitch = H; } else { src = h->enc[L].Hst + BP * h->esz; pitch = h->PH; }
  }
  else if (s == "h_t") { src = h->dec[L - 1].Hst + BP * h->esz; rows = T * Bp; cols = H; pitch = h->PH; isT = true; }
  else if (s == "att_a") { src = h->att_a; rows = 1; cols = pitch = T * Bp * S; }
  else if (s == "att_s") { src = h->att_s; rows = 1; cols = pitch = T * Bp * S; }
  else if ((s.rfind("enc.l", 0) == 0 || s.rfind("dec.l", 0) == 0) && s.size() >= 8) {
    // "<enc|dec>.l<k>[.fwd|.bwd].<h|c|gates>": states after every step and gate activations of one LSTM
    const bool enc = s[0] == 'e';
    size_t pos = 5;
    int l = 0;
    while (pos < s.size() && s[pos] >= '0' && s[pos] <= '9') l = l * 10 + (s[pos++] - '0');
    int dir = -1;
    if (s.compare(pos, 5, ".fwd.") == 0) { dir = 0; pos += 4; }
    else if (s.compare(pos, 5, ".bwd.") == 0) { dir = 1; pos += 4; }
    const std::string what = pos < s.size() ? s.substr(pos + 1) : "";
    if (l >= L || (what != "h" && what != "c" && what != "gates") || (dir >= 0) != (enc && l == 0))
      return fail(h, CMT_EINVAL, "unknown intermediate name");
    const LD& d = enc ? h->enc[l == 0 ? dir : l + 1] : h->dec[l];
    const size_t steps = enc ? S : T;
    // slot 0 of Hst / Cst holds the initial state (the reverse direction: slot S), slot t + 1 (reverse: t)
    // the state after the step at position t
    const size_t first = (enc && l == 0 && dir == 1) ? 0 : 1;
    rows = steps * Bp;
    if (what == "h") { src = d.Hst + first * Bp * d.ph * h->esz; cols = d.Hh; pitch = d.ph; isT = true; }
    else if (what == "c") { src = d.Cst + first * Bp * d.Hh; cols = pitch = d.Hh; }
    else { src = d.Gs; cols = pitch = 4 * (size_t)d.Hh; }
  }
  else if (s == "att_cs") { src = h->Cs; rows = T * Bp; cols = H; pitch = h->PH; isT = true; }
  else if (s == "h_o") { src = h->HoBuf + BP * h->esz; rows = T * Bp; cols = H; pitch = h->PH; isT = true; }
  else if (s == "h_o_drop") {
    src = (h->drop_p > 0.f ? h->HoDrop : h->HoBuf) + BP * h->esz; rows = T * Bp; cols = H; pitch = h->PH; isT = true;
  }
  else if (s == "lse" || s == "nll") {
    // kept per valid target position, densely numbered on the device: spread out to [T, Bp], zero elsewhere
    const size_t n = T * Bp;
    if (bytes != n * 4) return fail(h, CMT_EINVAL, "size mismatch for the requested intermediate");
    hipError_t e = hipStreamSynchronize(h->st);
    std::vector<int32_t> pos(n);
    std::vector<float> dense(n);
    if (e == hipSuccess) e = hipMemcpy(pos.data(), h->ce_pos, n * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(dense.data(), s == "lse" ? h->lse : h->nll, n * 4, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e, "cmt_debug_fetch");
    for (size_t i = 0; i < n; ++i) host_dst[i] = pos[i] >= 0 ? dense[pos[i]] : 0.f;
    return CMT_OK;
  }
  else return fail(h, CMT_EINVAL, "unknown intermediate name");
  const size_t n = rows * cols;
  if (bytes != n * 4) return fail(h, CMT_EINVAL, "size mismatch for the requested intermediate");
  hipError_t e = hipStreamSynchronize(h->st);
  if (e != hipSuccess) return hip_fail(h, e, "cmt_debug_fetch");
  if (isT && h->prec) {
    std::vector<uint16_t> tmp(n);
    e = hipMemcpy2D(tmp.data(), cols * 2, src, pitch * 2, cols * 2, rows, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e, "cmt_debug_fetch");
    for (size_t i = 0; i < n; ++i) { uint32_t u = ((uint32_t)tmp[i]) << 16; memcpy(&host_dst[i], &u, 4); }
  } else {
    e = hipMemcpy2D(host_dst, cols * 4, src, pitch * 4, cols * 4, rows, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e, "cmt_debug_fetch");
  }
  return CMT_OK;
}

const char* cmt_last_error(const cmt_handle* h) { return h ? h->err.c_str() : "null handle"; }

}  // extern "C"
