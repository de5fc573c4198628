// Host side of the Pacer hot-path library: argument validation, per-sequence bookkeeping and
// kernel sequencing for the C ABI declared in include/pacer.h.  No device memory is allocated
// here; everything lives in buffers the caller binds.
#include "../../include/pacer.h"
#include "kernels.h"
#include "kernels_w16.h"
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

namespace {

constexpr int kChunkRows = 32;       // rows of one sequence slot in a launch (two MFMA row tiles: what attention takes)
constexpr int kPrefillRows = PK_MAXB * kChunkRows;   // a prompt goes through the models 512 rows at a time
constexpr int kMaxChunks = 64;       // attention: key chunks per (head, sequence)
constexpr int kProfEvents = 32768;

struct Model {
  pacer_model_cfg cfg{};
  const void* embed = nullptr;
  const float* final_norm = nullptr;
  const void* head = nullptr;
  std::vector<const float*> attn_norm, ffn_norm;
  std::vector<const void*> wqkv, wo, wgu, wd;
  const float* posemb = nullptr;
  const float* cls = nullptr;
  void* kv = nullptr;
};

struct Seq {
  int len = 0;        // committed tokens
  int gamma = 0;      // drafts made in the current step
  int mb_done = 0;    // drafts already covered by pre-verification calls
  int verified = -1;  // gamma used by the last pacer_verify of this step, -1 = none
  float t = 0.f;      // current threshold
  bool pending = false;
  bool in_step = false;
  bool broken = false;   // a token id outside the vocabulary was met on the device: closed until the next prefill
  int last_n = -1, last_z = -1;
  int pv_ticket = 0;   // number of the last pre-verification call that covered this sequence (the kernel echoes it next to the stop flag)
  int acc_ticket = 0;  // number of the last accept call that covered it
  int force = -1;      // stop flag forced on the next pre-verification call (test tap): -1 none, 0 go on, 1 stop
  // the pending accept call, kept until its result is collected: what the bonus-row phase needs if every draft was accepted
  int acc_mode = 0, acc_slot = 0;
  float acc_beta = 0.f;
  uint64_t acc_seed = 0, acc_ctr = 0;
  const float* acc_logits = nullptr;
  int *acc_n = nullptr, *acc_z = nullptr;
};

}  // namespace

struct pacer_ctx {
  Model m[3];
  pacer_pv_cfg pv{};
  int max_batch = 0;
  hipStream_t stream = nullptr;
  Seq seq[PACER_MAX_BATCH];
  char err[256] = {0};
  // workspace carve-up
  bool ws_bound = false;
  int G1 = 0, rcap = 0, prows = 0, dmax = 0, fmax = 0, kmax = 0, hmax = 0, hdmax = 0, max_seq = 0;   // prows: rows the attention partials hold
  int *tokens = nullptr, *draft_tok = nullptr, *rej = nullptr;
  float* acc_part = nullptr;   // acceptance: per (slot, row, vocabulary chunk) statistics and candidates
  float *ring = nullptr, *hidden = nullptr, *x = nullptr, *xn = nullptr, *qkv = nullptr, *ao = nullptr, *gu = nullptr,
        *rope = nullptr, *part = nullptr;
  float* rope_pos[2] = {nullptr, nullptr};   // bf16 path: cos/sin of every position, [0] target, [1] draft and M_B (same head size and theta); filled at bind time
  _Float16 *xpA = nullptr, *xpB = nullptr, *qp = nullptr;   // bf16 path: ping-pong f16 operands, attention Q operand
  u64* ssq = nullptr;                                         // bf16 path: row sums of squares, [2*Lmax+1][rcap]
  float* pick_val = nullptr;                                  // bf16 path: per (row, vocab tile) token candidates
  int* pick_idx = nullptr;
  float* sk_part = nullptr;                                   // bf16 path: partial tiles of GEMMs whose K is split across blocks
  size_t sk_part_floats = 0;
  unsigned* sk_cnt = nullptr;                                 // their arrival counters (zero between launches)
  unsigned* att_cnt = nullptr;                                // attention key splits: arrival counters per (slot, head, row-tile half)
  int lmax = 0;
  // pinned host memory the kernels write and the host polls: [0..31] (n, z) per sequence, [32..47] accept
  // tickets, [48..63] stop flags with their tickets
  int* host_res = nullptr;
  int* host_res_dev = nullptr;  // its device alias
  int pv_calls = 0, acc_calls = 0;
  int64_t n_launches = 0;      // kernels enqueued so far
  // bf16 path: the last kernel of a draft step (or of a single-sequence pre-verification call) has already
  // written the embedding of the next draft step's input; valid only if exactly that step comes next
  bool pre_valid = false;
  int pre_n = 0, pre_seq[PACER_MAX_BATCH] = {0}, pre_j[PACER_MAX_BATCH] = {0};
  bool hip_failed = false;     // a HIP call failed since the hand-over counters were last cleared
  // profiling of the GEMM kernel
  bool prof = false;
  std::vector<hipEvent_t> ev;
  hipEvent_t pe0 = nullptr, pe1 = nullptr;   // the pair the next GEMM launch fills (null: launch untimed)
  int n_ev = 0;
  double prof_bytes = 0.0;
};

namespace {
// one word per sequence in pinned host memory (device alias): set by a kernel that met a token id outside the vocabulary
inline int* host_bad_dev(pacer_ctx* c) { return c->host_res_dev + 4 * PACER_MAX_BATCH; }
}  // namespace

namespace {

int fail(pacer_ctx* c, int code, const char* fmt, ...) {
  if (c) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

// every kernel launch of a context goes through these: the context counts its launches (pacer_launch_count)
#define PACER_LAUNCH(...) do { ++c->n_launches; hipLaunchKernelGGL(__VA_ARGS__); } while (0)
#define PACER_LAUNCH_EXT(...) do { ++c->n_launches; hipExtLaunchKernelGGL(__VA_ARGS__); } while (0)

// a HIP failure may have left a launch half done: its arrival counters are cleared again at the next step's start
#define HIPCHK(c, call)                                                                    \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess) {                                                                \
      if (c) (c)->hip_failed = true;                                                       \
      return fail(c, PACER_EHIP, "%s: %s", #call, hipGetErrorString(e_));                  \
    }                                                                                      \
  } while (0)

size_t esize(int dtype) { return dtype == PACER_BF16 ? 2 : 4; }

bool cfg_ok(const pacer_model_cfg& m) {
  if (m.n_layers < 1 || m.d_model < 1 || m.n_heads < 1 || m.d_ffn < 1 || m.vocab < 1 || m.max_seq < 2) return false;
  if (m.head_dim != 64 && m.head_dim != 128) return false;
  if (m.n_heads * m.head_dim != m.d_model) return false;
  if (m.dtype != PACER_F32 && m.dtype != PACER_BF16) return false;
  if (m.dtype == PACER_BF16 && (m.d_model % 32 || m.d_ffn % 32 || m.vocab % 16 || m.max_seq % 32)) return false;
  if (m.d_model % 8 || m.d_ffn % 8) return false;
  if (!(m.rms_eps > 0.f) || !(m.rope_theta > 0.f)) return false;
  if (m.dtype == PACER_F32 && m.head_dim != 64) return false;  // f32 KV tiles are staged for head_dim 64 only
  return true;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Carve {
  size_t off = 0;
  char* base;
  explicit Carve(void* b) : base(static_cast<char*>(b)) {}
  template <typename T> T* take(size_t n) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off = align_up(off + n * sizeof(T), 256);
    return p;
  }
};

// K split across blocks (few-tile GEMMs of the target): room for the partial tiles and the counters
constexpr size_t kSplitPartFloats = (size_t)1 << 20;   // 4 MiB: blocks x tiles per block x row tiles x 256 floats
constexpr int kSplitGroups = 512;

size_t carve(pacer_ctx* c, void* base) {
  Carve k(base);
  const int B = c->max_batch, G1 = c->G1, V = c->m[PACER_DRAFT].cfg.vocab, dD = c->m[PACER_DRAFT].cfg.d_model;
  const int mtcap = (c->rcap + 15) / 16;
  c->tokens = k.take<int>((size_t)B * c->max_seq);
  c->draft_tok = k.take<int>((size_t)B * G1);
  c->acc_part = k.take<float>((size_t)B * G1 * ACC_CHUNKS * ACC_PART);
  c->rej = k.take<int>((size_t)B * G1);
  c->ring = k.take<float>((size_t)B * G1 * V);
  c->hidden = k.take<float>((size_t)B * G1 * dD);
  c->x = k.take<float>((size_t)c->rcap * c->dmax);
  c->xn = k.take<float>((size_t)c->rcap * c->kmax);
  c->qkv = k.take<float>((size_t)c->rcap * 3 * c->dmax);
  c->ao = k.take<float>((size_t)c->rcap * c->dmax);
  c->gu = k.take<float>((size_t)c->rcap * 2 * c->fmax);
  c->rope = k.take<float>((size_t)c->rcap * c->hdmax);
  for (int w = 0; w < 2; ++w) c->rope_pos[w] = k.take<float>((size_t)c->max_seq * c->m[w].cfg.head_dim);
  c->part = k.take<float>((size_t)c->prows * c->hmax * kMaxChunks * (c->hdmax + 2));
  c->xpA = k.take<_Float16>((size_t)(c->kmax / 8 + 4) * mtcap * 16 * 8 * 2);      // hi and lo tiles
  c->xpB = k.take<_Float16>((size_t)(c->kmax / 8 + 4) * mtcap * 16 * 8 * 2);
  c->qp = k.take<_Float16>((size_t)PK_MAXB * (c->dmax / 32) * 2 * 1024);           // one slot per sequence slot of a launch
  c->ssq = k.take<u64>((size_t)(2 * c->lmax + 1) * SSQ_SUB * c->rcap);
  c->pick_val = k.take<float>((size_t)c->max_batch * (V / 16 + 1));
  c->pick_idx = k.take<int>((size_t)c->max_batch * (V / 16 + 1));
  // streaming kernel: kSplitPartFloats; wide kernel with K slices: up to 3 slices x padded rows x padded outputs (d wide)
  c->sk_part_floats = std::max(kSplitPartFloats, (size_t)3 * (c->rcap + 32) * (c->dmax + 128));
  c->sk_part = k.take<float>(c->sk_part_floats);
  c->sk_cnt = k.take<unsigned>(kSplitGroups);
  c->att_cnt = k.take<unsigned>((size_t)PK_MAXB * c->hmax * 2);
  return k.off;
}

Model* model_of(pacer_ctx* c, int which) { return (which >= 0 && which <= 2) ? &c->m[which] : nullptr; }

bool model_bound(const Model& m, int which) {
  if (!m.kv) return false;
  for (int l = 0; l < m.cfg.n_layers; ++l)
    if (!m.attn_norm[l] || !m.ffn_norm[l] || !m.wqkv[l] || !m.wo[l] || !m.wgu[l] || !m.wd[l]) return false;
  if (!m.final_norm) return false;
  if (which == PACER_PREVERIFY) return m.posemb && m.cls;
  return m.embed && m.head;
}

int ready(pacer_ctx* c) {
  if (!c->ws_bound) return fail(c, PACER_ESTATE, "workspace not bound");
  for (int w = 0; w < 3; ++w)
    if (!model_bound(c->m[w], w)) return fail(c, PACER_ESTATE, "model %d: weights or KV cache not bound", w);
  return PACER_OK;
}

int check_seqs(pacer_ctx* c, const int32_t* seqs, int n) {
  if (!seqs || n < 1 || n > c->max_batch) return fail(c, PACER_EINVAL, "bad sequence list (n_seqs=%d)", n);
  for (int i = 0; i < n; ++i) {
    if (seqs[i] < 0 || seqs[i] >= c->max_batch) return fail(c, PACER_EINVAL, "sequence id %d out of range", seqs[i]);
    for (int j = 0; j < i; ++j)
      if (seqs[j] == seqs[i]) return fail(c, PACER_EINVAL, "sequence id %d listed twice", seqs[i]);
  }
  return PACER_OK;
}

// ---- launches -------------------------------------------------------------------------------

// Kernel timing: the next launch of a GEMM kernel gets a pair of events that receive the kernel's own begin and end
// time stamps (hipExtLaunchKernelGGL), so a bracketed launch runs exactly as an unbracketed one: events recorded
// around a launch put two more packets into the queue and measure 2 us more than the kernel takes.
void prof_begin(pacer_ctx* c) {
  const bool on = c->prof && c->n_ev + 2 <= (int)c->ev.size();
  c->pe0 = on ? c->ev[c->n_ev] : nullptr;
  c->pe1 = on ? c->ev[c->n_ev + 1] : nullptr;
}
void prof_end(pacer_ctx* c, double bytes) {
  if (c->pe0) {
    c->n_ev += 2;
    c->prof_bytes += bytes;
  }
  c->pe0 = c->pe1 = nullptr;
}

bool is_w16(const Model& m) { return m.cfg.dtype == PACER_BF16; }
u64* slot(pacer_ctx* c, int s) { return c->ssq + (size_t)s * SSQ_SUB * c->rcap; }

// ===== bf16-weight path: fused GEMM epilogues, MFMA attention ================================

template <int EPI, int TAG, int HL, int MT, int NT, int WAVES, int U, int X17 = 0, int KSB = 1>
void launch_w16(pacer_ctx* c, GemmArgs ga, int n_tiles) {
  ga.sk_part = c->sk_part;
  ga.sk_cnt = c->sk_cnt;
  PACER_LAUNCH_EXT((gemm_w16_kernel<EPI, MT, NT, WAVES, U, TAG, X17, HL, KSB>), dim3((n_tiles + NT - 1) / NT * KSB), dim3(WAVES * 64), 0, c->stream, c->pe0,
                        c->pe1, 0, ga);
}

// Few-tile matrices of the target (O and down projections: about as many output tiles as CUs): tiles per
// block and K slices across blocks.  Every block fetches the operand rows of its K range, so with one
// tile per block the operand crosses L2 -> L1 once per tile, and a block count just above the CU count
// (320 or 448 tiles) takes two rounds.  The estimate counts what occupies the CU's outstanding-line
// capacity (about 128 lines): a weight line for ~1500 cycles (from HBM), an operand line for ~600 (from
// L2), on the busiest CU, plus the exchange of the partial sums.  Measured at 2.4 GHz, hi+lo operand:
//   7B down (256 tiles, K 11008), 17 rows: 1x1 25.4 us, 2x2 21.4, 4x4 21.5; 5 rows 19.6 / 17.7 / 19.7
//   13B down (320 tiles, K 13824), 13 rows: 1x1 47.7, 2x1 34.8, 4x2 31.4, 4x3 25.8
//   33B down (448 tiles, K 19200), 13 rows: 1x1 69.5, 2x1 52.2, 4x2 47.0; 17 rows 79.0 / 57.2 / 49.3
// (QKV and gate/up, with three or more tiles per block already, do not gain.)
struct SplitShape { int nt, ksb; };
SplitShape pick_split_shape(int n_tiles, int KT, int rows, int hl) {
  static const SplitShape cands[] = {{1, 1}, {2, 1}, {2, 2}, {3, 2}, {4, 2}, {4, 3}};
  static const double exchange_us[] = {0.0, 0.0, 1.5, 2.5};
  SplitShape best{1, 1};
  double best_us = 1e300;
  const double x_lines = hl * ((rows + 1) / 2);
  for (const SplitShape& s : cands) {
    const int blocks = (n_tiles + s.nt - 1) / s.nt * s.ksb;
    const int rounds = (blocks + 255) / 256;
    const double steps = (double)((KT + s.ksb - 1) / s.ksb);
    const double us = rounds * steps * (s.nt * 8 * 1500.0 + x_lines * 600.0) / 128.0 / 2400.0 + exchange_us[s.ksb];
    if (us < best_us) { best_us = us; best = s; }
  }
  return best;
}

// More than 32 rows: one launch of the wide kernel (operand shared through LDS, weights read once).
// K slices hand their sums over through the operand buffers: do they fit?
constexpr bool wide_fits(int hl, int mtb, int ntw, int ks) {
  return ks == 1 || 4 * ntw * mtb <= ks * 2 * (4 / ks) * ((mtb * hl + 3) / 4) * 4;
}
template <int EPI, int TAG, int HL, int MTB, int NTW, int KS>
void launch_wide_shape(pacer_ctx* c, const GemmArgs& ga, int n_tiles, int row_groups) {
  if constexpr (!wide_fits(HL, MTB, NTW, KS)) {
    (void)fail(c, PACER_EINVAL, "wide GEMM shape %d x %d with %d K slices does not exist", NTW, MTB, KS);
    return;
  } else {
  const int n_groups = (n_tiles + 4 * NTW - 1) / (4 * NTW);
  const dim3 grid((unsigned)((n_groups + 7) / 8 * 8 * row_groups));
  PACER_LAUNCH_EXT((gemm_wide_kernel<EPI, NTW, MTB, HL, TAG, KS>), grid, dim3(256 * KS), 0, c->stream, c->pe0, c->pe1, 0, ga, n_tiles, n_groups, row_groups);
  }
}
// Shape of a wide launch: row tiles per block (MTB), output tiles per wave (NTW), K slices (KS).
// A block always multiplies MTB row tiles (a short group repeats its last tile).  The launch moves
//   row_groups x weights  +  blocks x (the block's operand rows)
// through the L2s, which is what bounds it (about 12 TB/s measured), and it is only as fast as its busiest
// CU, so the estimate is that traffic times ceil(blocks / 256) / (blocks / 256).  Checked against
// microbenchmarks of the 13B-width matrices at 96..272 rows (random data): the estimate ranks the shapes
// as measured (e.g. QKV at 144 rows: 3 tiles x 3 row tiles = 240 blocks 61 us, 4 x 4 = 180 blocks 91 us; at
// 160 rows 3 x 4 = 240 blocks 74 us, 3 x 3 = 320 blocks 105 us).  Up to 256 blocks: two K slices of waves
// per block (8 waves on the CU); up to 128 blocks of one tile per wave: four.
struct WideShape { int mtb, ntw, ks; };
WideShape pick_wide_shape(int n_tiles, int mt_total, int KT, int hl) {
  WideShape best{4, 2, 1};
  double best_est = 1e300;
  for (int mtb = 3; mtb <= 4; ++mtb) {
    const int rg = (mt_total + mtb - 1) / mtb;
    for (int ntw = 1; ntw <= 4; ++ntw) {
      const int blocks = (n_tiles + 4 * ntw - 1) / (4 * ntw) * rg;
      int ks = 1;
      if (blocks <= 128 && ntw == 1 && KT % 16 == 0) ks = 4;
      else if (blocks <= 256 && KT % 8 == 0) ks = 2;
      if (!wide_fits(hl, mtb, ntw, ks)) ks = 1;
      if (ks == 1 && ntw == 1) continue;              // one tile per wave exists only with K slices
      const double traffic = (double)rg * n_tiles * 32.0 + (double)blocks * mtb * 64.0;
      const double est = traffic * ((blocks + 255) / 256) * 256.0 / blocks;
      if (est < best_est * 0.999 || (est < best_est * 1.001 && ntw > best.ntw)) { best_est = est; best = {mtb, ntw, ks}; }
    }
  }
  return best;
}
// Few-tile projections at 6..12 row tiles (96..192 rows: batched verification): the 8-wave kernel with K
// slices across blocks.  Two row groups of MTB = ceil(row tiles / 2) tiles, one output tile per wave, and as
// many K slices (3, else 2) as keep the launch within the CU count.  Measured at d 5120 (320 tiles -> 40 groups x
// 2 x 3 = 240 blocks), hi+lo down projection: 52 / 63 / 74 us at MTB 4 / 5 / 6 against 75 / 80 / 84 us for the best
// shape of the 4-wave kernel.  The hi-only O projection (26 / 31.5 us at MTB 4 / 5 against 31 / 33 us in the same
// microbenchmark) turned out slower in the real sequence (33 against 29 us) and stays with the 4-wave kernel.
// Returns false if the shape is not covered (the caller then takes the 4-wave kernel).
constexpr int kWide8KC = 4;
// The gate/up GEMM (many tiles) takes the same kernel without K slices at 7..12 row tiles when two tiles per
// wave x two row groups give 192..256 blocks (d 5120: 108 groups -> 216 blocks): 82 / 106 / 117 us at MTB 4 / 5 / 6
// against 88 / 115 / 123 us.  The QKV GEMM does not gain (94 against 62 us).
template <int EPI, int TAG, int HL, int NTW, int MTB, int KSB>
void launch_wide8_shape(pacer_ctx* c, const GemmArgs& ga, int n_tiles, int n_groups) {
  const size_t lds = (size_t)2 * kWide8KC * MTB * HL * 1024;
  PACER_LAUNCH_EXT((gemm_wide8_kernel<EPI, NTW, MTB, HL, TAG, kWide8KC, KSB>), dim3((unsigned)((n_groups + 7) / 8 * 8 * 2 * KSB)), dim3(512), lds,
                        c->stream, c->pe0, c->pe1, 0, ga, n_tiles, n_groups, 2);
}
template <int EPI, int TAG, int HL>
bool launch_wide8(pacer_ctx* c, GemmArgs ga, int n_tiles) {
  if constexpr (TAG == 0 && EPI == EPI_SWIGLU && HL == 2) {
    const int mt = ga.mt_total;
    const int n_groups = (n_tiles + 15) / 16;
    if (mt < 7 || mt > 12 || ga.KT % 4 || ga.KT < 64 || n_groups * 2 < 192 || n_groups * 2 > 256) return false;
    const int mtb = std::max(4, (mt + 1) / 2);
    ga.mt0 = 0;
    if (mtb == 4) launch_wide8_shape<EPI, TAG, HL, 2, 4, 1>(c, ga, n_tiles, n_groups);
    else if (mtb == 5) launch_wide8_shape<EPI, TAG, HL, 2, 5, 1>(c, ga, n_tiles, n_groups);
    else launch_wide8_shape<EPI, TAG, HL, 2, 6, 1>(c, ga, n_tiles, n_groups);
    return true;
  } else if constexpr (TAG != 0 || EPI != EPI_RESID || HL != 2) {
    return false;
  } else {
    const int mt = ga.mt_total;
    if (mt < 6 || mt > 12 || n_tiles >= 512 || ga.KT % 4 || ga.KT < 64) return false;
    const int n_groups = (n_tiles + 7) / 8;
    const int mtb = std::max(4, (mt + 1) / 2);
    const int ksb = n_groups * 2 * 3 <= 256 ? 3 : (n_groups * 2 * 2 <= 256 ? 2 : 0);
    if (ksb == 0 || n_groups * 2 > kSplitGroups) return false;
    if ((size_t)n_groups * 2 * ksb * 8 * mtb * 256 > c->sk_part_floats) return false;
    ga.mt0 = 0;
    ga.sk_part = c->sk_part;
    ga.sk_cnt = c->sk_cnt;
#define PACER_W8(MTB_) if (ksb == 3) launch_wide8_shape<EPI, TAG, HL, 1, MTB_, 3>(c, ga, n_tiles, n_groups); else launch_wide8_shape<EPI, TAG, HL, 1, MTB_, 2>(c, ga, n_tiles, n_groups)
    if (mtb == 4) { PACER_W8(4); } else if (mtb == 5) { PACER_W8(5); } else { PACER_W8(6); }
#undef PACER_W8
    return true;
  }
}

template <int EPI, int TAG, int HL>
void launch_wide(pacer_ctx* c, GemmArgs ga, int n_tiles) {
  ga.mt0 = 0;
  if constexpr (TAG != 0) {   // draft and pre-verification layer: small matrices, one shape
    launch_wide_shape<EPI, TAG, HL, 4, 2, 1>(c, ga, n_tiles, (ga.mt_total + 3) / 4);
  } else {
    const WideShape w = pick_wide_shape(n_tiles, ga.mt_total, ga.KT, HL);
    const int rg = (ga.mt_total + w.mtb - 1) / w.mtb;
#define PACER_WIDE(MTB_, NTW_, KS_) launch_wide_shape<EPI, TAG, HL, MTB_, NTW_, KS_>(c, ga, n_tiles, rg)
#define PACER_WIDE_MTB(MTB_)                                                     \
    if (w.ks == 4) PACER_WIDE(MTB_, 1, 4);                                       \
    else if (w.ks == 2) {                                                        \
      if (w.ntw == 1) PACER_WIDE(MTB_, 1, 2); else if (w.ntw == 2) PACER_WIDE(MTB_, 2, 2); \
      else if (w.ntw == 3) PACER_WIDE(MTB_, 3, 2); else PACER_WIDE(MTB_, 4, 2);  \
    } else {                                                                     \
      if (w.ntw == 2) PACER_WIDE(MTB_, 2, 1); else if (w.ntw == 3) PACER_WIDE(MTB_, 3, 1); \
      else PACER_WIDE(MTB_, 4, 1);                                               \
    }
    if (w.mtb == 3) { PACER_WIDE_MTB(3) } else { PACER_WIDE_MTB(4) }
#undef PACER_WIDE_MTB
#undef PACER_WIDE
  }
}

// Launches the GEMM over `n_tiles` output tiles starting at ga.nt_begin; up to 32 rows with the
// weight-streaming kernel, more with the wide one.
// HL = 2: multiply the operand's hi and lo tiles (target model, all GEMMs but the O projection and the
// LM head, whose inputs' f16 rounding hardly shows in the logits); HL = 1: hi only.
// Launch shapes <MT, NT, WAVES, U>, all measured on MI355X (U = K steps per register set; the loop keeps
// two sets in flight, so one or two steps per set is enough).  Few tiles (O and down projections): 8 waves
// split K, one tile per block, held to 128 VGPRs so that two blocks fit a CU.  Many tiles: the waves of a
// block share an operand fetch among NT tiles; HL = 2 doubles the operand traffic from L2, which becomes
// the limiter as rows grow.  17 rows exactly (full window + committed token): the second row tile is
// reduced to its one live column (X17).
// TAG gives the target model's launches their own kernel symbols; the GEMM profile counts those.
template <int EPI, int TAG, int HL>
void gemm_w16_tag(pacer_ctx* c, GemmArgs ga, int n_tiles, int K) {
  const int mt_total = (ga.R + 15) / 16;
  ga.mt_total = mt_total;
  ga.KT = K / 32;
  ga.nt_end = ga.nt_begin + n_tiles;
  const bool many = n_tiles >= 512;
  const bool even = n_tiles % 2 == 0;
  if (mt_total > 2 && ga.KT % 4 == 0) {
    if (TAG == 0) prof_begin(c);
    if (!launch_wide8<EPI, TAG, HL>(c, ga, n_tiles)) launch_wide<EPI, TAG, HL>(c, ga, n_tiles);
    if (TAG == 0) prof_end(c, (double)n_tiles * 16.0 * K * 2.0);
    return;
  }
  for (int mt0 = 0; mt0 < mt_total; mt0 += 2) {
    const int mt = std::min(2, mt_total - mt0);
    const int rows = ga.R - 16 * mt0;
    ga.mt0 = mt0;
    if (TAG == 0) prof_begin(c);
    if constexpr (TAG == 0 && EPI == EPI_RESID) {
      const SplitShape sp = (!many && ga.KT >= 64) ? pick_split_shape(n_tiles, ga.KT, std::min(rows, 32), HL) : SplitShape{1, 1};
      const size_t part_floats = (size_t)((n_tiles + sp.nt - 1) / sp.nt) * sp.ksb * sp.nt * mt * 256;
      if (sp.nt > 1 && part_floats <= kSplitPartFloats && (n_tiles + sp.nt - 1) / sp.nt <= kSplitGroups) {
#define PACER_SPLIT(NT_, KSB_)                                                                       \
        if (mt == 1) launch_w16<EPI, TAG, HL, 1, NT_, 8, 1, 0, KSB_>(c, ga, n_tiles);                \
        else if (rows == 17) launch_w16<EPI, TAG, HL, 2, NT_, 8, 1, 1, KSB_>(c, ga, n_tiles);        \
        else launch_w16<EPI, TAG, HL, 2, NT_, 8, 1, 0, KSB_>(c, ga, n_tiles)
        if (sp.nt == 2 && sp.ksb == 1) { PACER_SPLIT(2, 1); }
        else if (sp.nt == 2) { PACER_SPLIT(2, 2); }
        else if (sp.nt == 3) { PACER_SPLIT(3, 2); }
        else if (sp.ksb == 2) { PACER_SPLIT(4, 2); }
        else { PACER_SPLIT(4, 3); }
#undef PACER_SPLIT
        prof_end(c, (double)n_tiles * 16.0 * K * 2.0);
        continue;
      }
    }
    if (HL == 1) {
      if (mt == 1) {
        // K <= 768 (draft, pre-verification layer): 4 waves with at most 6 K steps each; the LM head and the
        // gate/up matrix (many tiles) run one step per register set, the small ones three
        if (ga.KT <= 24) {
          if (n_tiles >= 256) launch_w16<EPI, TAG, 1, 1, 1, 4, 1>(c, ga, n_tiles);
          else launch_w16<EPI, TAG, 1, 1, 1, 4, 3>(c, ga, n_tiles);
        } else if (many && even && rows > 8) launch_w16<EPI, TAG, 1, 1, 2, 4, 2>(c, ga, n_tiles);
        else launch_w16<EPI, TAG, 1, 1, 1, 8, 2>(c, ga, n_tiles);
      } else if (rows == 17) {
        if (many && even && n_tiles >= 1024) launch_w16<EPI, TAG, 1, 2, 2, 4, 2, 1>(c, ga, n_tiles);
        else if (many) launch_w16<EPI, TAG, 1, 2, 1, 4, 4, 1>(c, ga, n_tiles);
        else launch_w16<EPI, TAG, 1, 2, 1, 8, 2, 1>(c, ga, n_tiles);
      } else {
        if (many && even) launch_w16<EPI, TAG, 1, 2, 2, 4, 4>(c, ga, n_tiles);
        else launch_w16<EPI, TAG, 1, 2, 1, 8, 2>(c, ga, n_tiles);
      }
    } else {
      // Output tiles per wave (NT): a wave's tiles share one fetch of the operand, so more is better, but the
      // launch is only as fast as its busiest CU.  Cost model: ceil(blocks / 256) * NT with blocks =
      // ceil(tiles / NT) (the last block may overhang).  Ties go to the shape with at most one block per CU
      // (each CU then fetches the operand once), else to two tiles for very wide matrices, else to the larger NT.
      // 7B QKV, 768 tiles: NT 3 = 256 blocks 17 us, NT 4 = 192 blocks 19.5 us, NT 2 = 384 blocks 21 us.
      // 7B gate/up, 1376 tiles, 13 rows: NT 6 = 230 blocks 29.7 us (the weights-only time), NT 2 = 688 blocks 33.6 us.
      int nt = 1;
      if (many) {
        int best = 1 << 30;
        bool best_single = false;
        for (int cand : {2, 3, 4, 6, 7}) {
          if (cand > 4 && rows <= 8) break;              // up to 8 rows the operand is small and more blocks stream better
          const int blocks = (n_tiles + cand - 1) / cand;
          const int units = (blocks + 255) / 256 * cand;
          const bool single = blocks <= 256;
          bool take = units < best;
          if (units == best) take = single ? !best_single : (!best_single && n_tiles < 1024);   // candidates come in increasing order
          if (take) { best = units; nt = cand; best_single = single; }
        }
      }
      if (mt == 1) {
        if (nt == 7) launch_w16<EPI, TAG, 2, 1, 7, 8, 1>(c, ga, n_tiles);
        else if (nt == 6) launch_w16<EPI, TAG, 2, 1, 6, 8, 1>(c, ga, n_tiles);
        else if (nt == 4) launch_w16<EPI, TAG, 2, 1, 4, 8, 1>(c, ga, n_tiles);
        else if (nt == 3) launch_w16<EPI, TAG, 2, 1, 3, 8, 1>(c, ga, n_tiles);
        else if (nt == 2) launch_w16<EPI, TAG, 2, 1, 2, 4, 4>(c, ga, n_tiles);
        else launch_w16<EPI, TAG, 2, 1, 1, 8, 1>(c, ga, n_tiles);
      } else if (rows == 17) {
        if (nt == 7) launch_w16<EPI, TAG, 2, 2, 7, 8, 1, 1>(c, ga, n_tiles);
        else if (nt == 6) launch_w16<EPI, TAG, 2, 2, 6, 8, 1, 1>(c, ga, n_tiles);
        else if (nt == 4) launch_w16<EPI, TAG, 2, 2, 4, 8, 1, 1>(c, ga, n_tiles);
        else if (nt == 3) launch_w16<EPI, TAG, 2, 2, 3, 8, 1, 1>(c, ga, n_tiles);
        else if (nt == 2) launch_w16<EPI, TAG, 2, 2, 2, 4, 2, 1>(c, ga, n_tiles);
        else launch_w16<EPI, TAG, 2, 2, 1, 8, 1, 1>(c, ga, n_tiles);
      } else {
        if (many && even) launch_w16<EPI, TAG, 2, 2, 2, 4, 2>(c, ga, n_tiles);
        else launch_w16<EPI, TAG, 2, 2, 1, 8, 2>(c, ga, n_tiles);
      }
    }
    if (TAG == 0) prof_end(c, (double)n_tiles * 16.0 * K * 2.0);
  }
}
template <int EPI>
void gemm_w16(pacer_ctx* c, int tag, bool hilo, const GemmArgs& ga, int n_tiles, int K) {
  if (tag == 0) {
    // the target's QKV and gate/up GEMMs always take hi+lo, its LM head never does
    if constexpr (EPI == EPI_QKV || EPI == EPI_SWIGLU) gemm_w16_tag<EPI, 0, 2>(c, ga, n_tiles, K);
    else if constexpr (EPI == EPI_STORE) gemm_w16_tag<EPI, 0, 1>(c, ga, n_tiles, K);
    else if (hilo) gemm_w16_tag<EPI, 0, 2>(c, ga, n_tiles, K);
    else gemm_w16_tag<EPI, 0, 1>(c, ga, n_tiles, K);
  } else {
    gemm_w16_tag<EPI, 1, 1>(c, ga, n_tiles, K);
  }
}

void rope_table(pacer_ctx* c, const Model& m, int R, const SeqRows& sr) {
  PACER_LAUNCH(rope_table_kernel, dim3(R), dim3(m.cfg.head_dim / 2), 0, c->stream, sr, m.cfg.head_dim, m.cfg.rope_theta, c->rope);
}

// Decoder stack of a bf16 model on R rows.  On entry x holds the rows, xpA their f16 operand x*g of
// the first norm and slot 0 their sums of squares.  On exit (not kv_only) x holds the final residual
// rows, xpA = f16(x * g_final) and slot 2L their sums of squares.
// cache_only: the caller needs nothing but the KV cache rows (prompt ingestion of the target model), so the last
// layer stops after its keys and values.
void run_layers_w16(pacer_ctx* c, const Model& m, int tag, int R, const SeqRows& sr, bool kv_only, bool cache_only = false) {
  const pacer_model_cfg& g = m.cfg;
  const int d = g.d_model, F = g.d_ffn, L = g.n_layers, H = g.n_heads, hd = g.head_dim;
  const int mt_total = (R + 15) / 16;
  int max_keys = 0, max_rows = 0;
  for (int i = 0; i < sr.n_seqs; ++i) {
    max_keys = std::max(max_keys, sr.pos0[i] + sr.row_off[i + 1] - sr.row_off[i]);
    max_rows = std::max(max_rows, sr.row_off[i + 1] - sr.row_off[i]);
  }
  // Keys per block (8 waves).  One block per (head, sequence) writes its output itself; with the keys split
  // over several blocks the last one to finish combines the partial results (about 2 us for the hand-over).
  // A (head, sequence) pair's keys stream through one CU's outstanding-line capacity, so few pairs with
  // many keys want splits: never more blocks than CUs (544 blocks of 256 keys take twice as long as 160
  // blocks of 1024; 512 blocks of 540 keys make the 4k-context verify pass 8 % slower than 256), and no splits
  // below 512 keys.  Measured, 32 heads, one sequence, cold cache, 13 rows: 300 keys 6.9 us unsplit, 8.6 with 2
  // splits; 800 keys 13.4 / 10.3 (6 splits); 1600 keys 20.9 / 13.2 (8); 4300 keys 46.0 / 19.3 (8).  In the decode
  // loop at 770 keys, blocks of at least 96 / 128 / 160 keys (8 / 6 / 4 splits): verify pass 2.930 / 2.942 / 2.957 ms.
  int kps = (max_keys + 31) / 32 * 32;
  {
    const int pairs = H * sr.n_seqs;
    // (the small draft model's keys are re-read every few microseconds and sit in L2: 770 keys, 12 heads take
    // 6.6 us unsplit and 7.3 us in 4 splits, so its blocks keep at least 1024 keys)
    const int min_keys = tag == 0 ? (max_keys >= 512 ? 96 : 256) : 1024;
    const int most = std::min({256 / pairs, max_keys / min_keys, kMaxChunks});   // splits that still leave one block per CU
    // 17..32 rows below 1000 keys: two one-tile blocks per pair instead (see the attention launch)
    const bool two_tiles_short = max_rows > 16 && max_keys < 1000;
    if (most >= 2 && !two_tiles_short && R <= c->prows) kps = ((max_keys + most - 1) / most + 31) / 32 * 32;
  }
  const int S = (max_keys + kps - 1) / kps;
  GemmArgs base{};
  base.R = R;
  base.sr = sr;
  base.G1 = c->G1;
  base.rowmap = ROWMAP_ID;
  base.eps = g.rms_eps;
  base.ssq_stride = c->rcap;
  base.d = d; base.hd = hd; base.n_layers = L; base.max_seq = g.max_seq; base.H = H;
  base.mt_total_out = mt_total;
  for (int l = 0; l < L; ++l) {
    {
      GemmArgs ga = base;
      ga.W = static_cast<const u32x4*>(m.wqkv[l]);
      ga.X = reinterpret_cast<const u32x4*>(c->xpA);
      ga.ssq_in = slot(c, 2 * l);
      ga.inv_dim = 1.0f / d;
      ga.qp = c->qp;
      ga.kv = static_cast<_Float16*>(m.kv);
      ga.rope = c->rope_pos[tag == 0 ? PACER_TARGET : PACER_DRAFT];
      ga.layer = l;
      ga.nt_begin = kv_only ? d / 16 : 0;
      gemm_w16<EPI_QKV>(c, tag, true, ga, (kv_only ? 2 : 3) * d / 16, d);
    }
    if (kv_only || (cache_only && l + 1 == L)) continue;
    {
      const _Float16* kv = static_cast<const _Float16*>(m.kv);
      // 17..32 rows per sequence: two row tiles.  With a short context and few (head, sequence) pairs the
      // launch is a chain of memory latencies on a few dozen CUs, and the one-tile kernel run as two blocks
      // per pair, one per row tile, is faster than the two-tile kernel although it reads the keys twice
      // (7B shape, 550 keys, warm cache: 7.1 us against 10.0 us).  Long contexts and batches are bound by the
      // cache traffic and keep the two-tile kernel.
      const bool rt_split = max_rows > 16 && S == 1 && max_keys < 1000 && H * sr.n_seqs <= 64;
      const int mrows = rt_split ? 16 : max_rows;
      const dim3 grid(rt_split ? 2 * S : S, H, sr.n_seqs);
      // LDS for the wave states: 8 waves x live rows x (hd + 4) floats
#define PACER_ATT(HD_, MT_, QL_) PACER_LAUNCH((attn_mfma_kernel<HD_, MT_, QL_>), grid, dim3(512), (size_t)8 * std::min(mrows, MT_ * 16) * (HD_ + 4) * 4, c->stream, c->qp, kv, l, L, g.max_seq, d, sr, kps, S, H, c->part, c->xpB, mt_total, rt_split ? 1 : 0, c->att_cnt)
      if (tag == 0) {
        if (hd == 128) { if (mrows > 16) PACER_ATT(128, 2, 2); else PACER_ATT(128, 1, 2); }
        else           { if (mrows > 16) PACER_ATT(64, 2, 2); else PACER_ATT(64, 1, 2); }
      } else {
        if (hd == 128) { if (mrows > 16) PACER_ATT(128, 2, 1); else PACER_ATT(128, 1, 1); }
        else           { if (mrows > 16) PACER_ATT(64, 2, 1); else PACER_ATT(64, 1, 1); }
      }
#undef PACER_ATT
    }
    {
      GemmArgs ga = base;
      ga.W = static_cast<const u32x4*>(m.wo[l]);
      ga.X = reinterpret_cast<const u32x4*>(c->xpB);
      ga.out = c->x; ga.ldo = c->dmax;
      ga.g_next = m.ffn_norm[l];
      ga.xp_out = c->xpA;
      ga.ssq_out = slot(c, 2 * l + 1);
      gemm_w16<EPI_RESID>(c, tag, false, ga, d / 16, d);
    }
    {
      GemmArgs ga = base;
      ga.W = static_cast<const u32x4*>(m.wgu[l]);
      ga.X = reinterpret_cast<const u32x4*>(c->xpA);
      ga.ssq_in = slot(c, 2 * l + 1);
      ga.inv_dim = 1.0f / d;
      ga.xp_out = c->xpB;
      gemm_w16<EPI_SWIGLU>(c, tag, true, ga, 2 * F / 16, d);
    }
    {
      GemmArgs ga = base;
      ga.W = static_cast<const u32x4*>(m.wd[l]);
      ga.X = reinterpret_cast<const u32x4*>(c->xpB);
      ga.out = c->x; ga.ldo = c->dmax;
      ga.g_next = (l + 1 < L) ? m.attn_norm[l + 1] : m.final_norm;
      ga.xp_out = c->xpA;
      ga.ssq_out = slot(c, 2 * l + 2);
      gemm_w16<EPI_RESID>(c, tag, true, ga, d / 16, F);
    }
  }
}

// where a forward of model m on R rows expects its embedded input
EmbedOut embed_out(pacer_ctx* c, const Model& m, int R) {
  EmbedOut o{};
  o.x = c->x; o.ldx = c->dmax; o.g = m.attn_norm[0]; o.xp = c->xpA; o.MT_total = (R + 15) / 16;
  o.ssq = c->ssq; o.n_slots = 2 * m.cfg.n_layers + 1; o.slot_stride = c->rcap;
  return o;
}
void embed_w16(pacer_ctx* c, const Model& m, int R, const SeqRows& sr) {
  PACER_LAUNCH(embed_w16_kernel, dim3(R), dim3(256), 0, c->stream, static_cast<const uint16_t*>(m.embed), c->tokens, c->draft_tok, sr,
               c->max_seq, c->G1, m.cfg.d_model, embed_out(c, m, R));
}

struct PickCfg { int on, mode; uint64_t seed; uint32_t step; };

void lm_head_w16(pacer_ctx* c, const Model& m, int tag, int R, float* out, const SeqRows& sr, int rowmap, const PickCfg* pick = nullptr) {
  GemmArgs ga{};
  if (pick && pick->on) {
    ga.pick_val = c->pick_val;
    ga.pick_idx = c->pick_idx;
    ga.pick_tiles = m.cfg.vocab / 16;
    ga.pick_mode = pick->mode;
    ga.pick_seed = pick->seed;
    ga.pick_step = pick->step;
  }
  ga.R = R; ga.sr = sr; ga.G1 = c->G1; ga.rowmap = rowmap; ga.eps = m.cfg.rms_eps;
  ga.W = static_cast<const u32x4*>(m.head);
  ga.X = reinterpret_cast<const u32x4*>(c->xpA);
  ga.ssq_in = slot(c, 2 * m.cfg.n_layers);
  ga.ssq_stride = c->rcap;
  ga.inv_dim = 1.0f / m.cfg.d_model;
  ga.out = out; ga.ldo = m.cfg.vocab;
  gemm_w16<EPI_STORE>(c, tag, false, ga, m.cfg.vocab / 16, m.cfg.d_model);
}

// ===== f32 path (tiny pair): plain kernels, one per operation ================================

void gemm_f32(pacer_ctx* c, const void* W, const float* act, int lda, float* out, int ldo, int R, int N, int K, int acc,
              const SeqRows& sr, int rowmap) {
  PACER_LAUNCH(gemm_f32_kernel, dim3((N + 3) / 4), dim3(256), 0, c->stream, static_cast<const float*>(W), act, lda, out, ldo, R, N,
                     K, acc, sr, rowmap, c->G1);
}

void rmsnorm_f32(pacer_ctx* c, const Model& m, const float* g, int R, float* hid_out, const SeqRows& sr) {
  PACER_LAUNCH(rmsnorm_pack_kernel, dim3(R), dim3(256), 0, c->stream, c->x, c->dmax, g, m.cfg.rms_eps, R, m.cfg.d_model, c->xn,
                     c->kmax, hid_out, c->G1, sr);
}

void run_layers_f32(pacer_ctx* c, const Model& m, int R, const SeqRows& sr, bool kv_only, float* hid_out, bool cache_only = false) {
  const pacer_model_cfg& g = m.cfg;
  const int d = g.d_model, F = g.d_ffn, H = g.n_heads, hd = g.head_dim;
  const SeqRows none{};
  rope_table(c, m, R, sr);
  for (int l = 0; l < g.n_layers; ++l) {
    rmsnorm_f32(c, m, m.attn_norm[l], R, nullptr, sr);
    gemm_f32(c, m.wqkv[l], c->xn, c->kmax, c->qkv, 3 * c->dmax, R, 3 * d, d, 0, none, ROWMAP_ID);
    PACER_LAUNCH((rope_append_kernel<float>), dim3(R, H), dim3(hd / 2), 0, c->stream, c->qkv, 3 * c->dmax, c->rope, sr, d, hd,
                       static_cast<float*>(m.kv), l, g.n_layers, g.max_seq, kv_only ? 1 : 0);
    if (kv_only || (cache_only && l + 1 == g.n_layers)) continue;
    int max_keys = 0;
    for (int i = 0; i < sr.n_seqs; ++i) max_keys = std::max(max_keys, sr.pos0[i] + sr.row_off[i + 1] - sr.row_off[i]);
    const int n_tiles = (max_keys + ATT_TILE - 1) / ATT_TILE;
    int chunks = std::min(std::min(n_tiles, kMaxChunks), std::max(1, 1024 / (H * sr.n_seqs)));
    const int tpc = (n_tiles + chunks - 1) / chunks;
    chunks = (n_tiles + tpc - 1) / tpc;
    PACER_LAUNCH((attn_partial_kernel<float, 64>), dim3(chunks, H, sr.n_seqs), dim3(256), 0, c->stream, c->qkv, 3 * c->dmax,
                       static_cast<const float*>(m.kv), l, g.n_layers, g.max_seq, d, sr, tpc, chunks, H, c->part);
    PACER_LAUNCH(attn_combine_kernel, dim3(R, H), dim3(hd), 0, c->stream, c->part, chunks, H, hd, c->ao, c->dmax);
    gemm_f32(c, m.wo[l], c->ao, c->dmax, c->x, c->dmax, R, d, d, 1, none, ROWMAP_ID);
    rmsnorm_f32(c, m, m.ffn_norm[l], R, nullptr, sr);
    gemm_f32(c, m.wgu[l], c->xn, c->kmax, c->gu, 2 * c->fmax, R, 2 * F, d, 0, none, ROWMAP_ID);
    PACER_LAUNCH(swiglu_pack_kernel, dim3((F / 8 + 255) / 256, R), dim3(256), 0, c->stream, c->gu, 2 * c->fmax, R, F, c->xn, c->kmax);
    gemm_f32(c, m.wd[l], c->xn, c->kmax, c->x, c->dmax, R, d, F, 1, none, ROWMAP_ID);
  }
  if (!kv_only && !cache_only) rmsnorm_f32(c, m, m.final_norm, R, hid_out, sr);
}

// ===== model-level steps, both paths ==========================================================

// rows -> x (embedding gather) and the decoder stack; `tag` 0 = target model
void forward_lm(pacer_ctx* c, const Model& m, int tag, int R, const SeqRows& sr, bool cache_only = false) {
  c->pre_valid = false;      // x, the operand buffers and the sums of squares are about to be overwritten
  if (is_w16(m)) {
    embed_w16(c, m, R, sr);
    run_layers_w16(c, m, tag, R, sr, false, cache_only);
  } else {
    PACER_LAUNCH((embed_rows_kernel<float>), dim3(R), dim3(256), 0, c->stream, static_cast<const float*>(m.embed), c->tokens,
                       c->draft_tok, sr, c->max_seq, c->G1, m.cfg.d_model, c->x, c->dmax);
    run_layers_f32(c, m, R, sr, false, nullptr, cache_only);
  }
}

void lm_head(pacer_ctx* c, const Model& m, int tag, int R, float* out, const SeqRows& sr, int rowmap) {
  if (is_w16(m)) lm_head_w16(c, m, tag, R, out, sr, rowmap);
  else gemm_f32(c, m.head, c->xn, c->kmax, out, m.cfg.vocab, R, m.cfg.vocab, m.cfg.d_model, 0, sr, rowmap);
}

// M_B over rows whose inputs are src rows + PosEmb; kv_only for prefix rows.
void run_preverify_rows(pacer_ctx* c, int R, const SeqRows& sr, const MbRows& mr, const float* src, int lds, bool kv_only) {
  const Model& mb = c->m[PACER_PREVERIFY];
  c->pre_valid = false;
  if (is_w16(mb)) {
    PACER_LAUNCH(mb_input_w16_kernel, dim3(R), dim3(256), 0, c->stream, src, lds, mb.posemb, sr, mr, mb.cfg.d_model, c->x, c->dmax,
                       mb.attn_norm[0], c->xpA, (R + 15) / 16, c->ssq, 3, c->rcap);
    run_layers_w16(c, mb, 1, R, sr, kv_only);
  } else {
    PACER_LAUNCH(mb_input_kernel, dim3(R), dim3(256), 0, c->stream, src, lds, mb.posemb, sr, mr, mb.cfg.d_model, c->x, c->dmax);
    run_layers_f32(c, mb, R, sr, kv_only, nullptr);
  }
}

// the 2-class head, block mean and stop flag for n sequences of b rows each (after run_preverify_rows)
// next_tok (device, may be null): the newest draft token of the call's single sequence; the head kernel then also
// embeds it for the next round's first draft step
void preverify_head(pacer_ctx* c, int n, int b, const HaltArgs& ha, float* dev_alpha, int* dev_stop, const int* next_tok) {
  const Model& mb = c->m[PACER_PREVERIFY];
  const Model& md = c->m[PACER_DRAFT];
  if (is_w16(mb))
    PACER_LAUNCH(mb_head_w16_kernel, dim3(n), dim3(256), 0, c->stream, c->x, c->dmax, mb.final_norm, slot(c, 2), c->rcap, 1.0f / mb.cfg.d_model,
                 mb.cfg.rms_eps, mb.cls, mb.cfg.d_model, b, ha, dev_alpha, dev_stop, c->host_res_dev + 3 * PACER_MAX_BATCH,
                 next_tok ? static_cast<const uint16_t*>(md.embed) : nullptr, next_tok, embed_out(c, md, 1));
  else
    PACER_LAUNCH(mb_head_kernel, dim3(n), dim3(256), 0, c->stream, c->xn, c->kmax, mb.cls, mb.cfg.d_model, b, ha, dev_alpha, dev_stop,
                       c->host_res_dev + 3 * PACER_MAX_BATCH);
}

// one draft forward at draft index j[s] (0-based) for each listed sequence; logits and hidden
// state go to ring slot j, and a token is picked into draft_tok[j]
void draft_forward(pacer_ctx* c, const int32_t* seqs, int n, const int* j, int mode, uint64_t seed, uint64_t ctr) {
  const Model& md = c->m[PACER_DRAFT];
  SeqRows sr{};
  PickArgs pa{};
  sr.n_seqs = pa.n_seqs = n;
  for (int i = 0; i < n; ++i) {
    const Seq& s = c->seq[seqs[i]];
    sr.seq[i] = pa.seq[i] = seqs[i];
    sr.row_off[i] = i;
    sr.pos0[i] = s.len - 1 + j[i];
    sr.len[i] = s.len;
    pa.j[i] = j[i];
  }
  sr.row_off[n] = n;
  if (is_w16(md)) {
    // the previous draft step's last kernel (or the pre-verification head) has embedded this step's input already
    bool have = c->pre_valid && c->pre_n == n;
    for (int i = 0; have && i < n; ++i) have = c->pre_seq[i] == seqs[i] && c->pre_j[i] == j[i];
    c->pre_valid = false;
    if (!have) embed_w16(c, md, n, sr);
    run_layers_w16(c, md, 1, n, sr, false);
    const PickCfg pick{1, mode, seed, (uint32_t)ctr};
    lm_head_w16(c, md, 1, n, c->ring, sr, ROWMAP_RING, &pick);
    PACER_LAUNCH(draft_tail_kernel, dim3(n), dim3(256), 0, c->stream, c->x, c->dmax, md.final_norm, slot(c, 2 * md.cfg.n_layers),
                 c->rcap, 1.0f / md.cfg.d_model, md.cfg.rms_eps, md.cfg.d_model, c->hidden, c->pick_val, c->pick_idx, md.cfg.vocab / 16,
                 c->draft_tok, pa, c->G1, static_cast<const uint16_t*>(md.embed), embed_out(c, md, n), md.cfg.vocab, host_bad_dev(c));
    c->pre_valid = true;
    c->pre_n = n;
    for (int i = 0; i < n; ++i) { c->pre_seq[i] = seqs[i]; c->pre_j[i] = j[i] + 1; }
  } else {
    PACER_LAUNCH((embed_rows_kernel<float>), dim3(n), dim3(256), 0, c->stream, static_cast<const float*>(md.embed), c->tokens,
                       c->draft_tok, sr, c->max_seq, c->G1, md.cfg.d_model, c->x, c->dmax);
    run_layers_f32(c, md, n, sr, false, c->hidden);
    lm_head(c, md, 1, n, c->ring, sr, ROWMAP_RING);
    PACER_LAUNCH(pick_token_kernel, dim3(n), dim3(1024), 0, c->stream, c->ring, c->draft_tok, pa, c->G1, md.cfg.vocab, mode, seed,
                       (uint32_t)ctr, host_bad_dev(c));
  }
}

// Waits until the kernel-written word *p (pinned host memory) carries `ticket` (in its bits above `shift`).
// Polling costs a few microseconds where hipStreamSynchronize costs twenty to thirty; if the word does not
// arrive within the spin budget the stream is synchronised and the word checked once more.
int wait_ticket(pacer_ctx* c, const int* p, int ticket, int shift) {
  const volatile int* v = p;
  for (long spin = 0; spin < 200000000L; ++spin) {
    if ((*v >> shift) == ticket) { std::atomic_thread_fence(std::memory_order_acquire); return PACER_OK; }
    if ((spin & 1023) == 1023 && hipStreamQuery(c->stream) == hipSuccess) break;   // stream drained: the word is final
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if ((*v >> shift) == ticket) return PACER_OK;
  return fail(c, PACER_EHIP, "a kernel's result did not reach host memory (ticket %d, found %d)", ticket, *v >> shift);
}

// Has a kernel reported, for sequence s, a token id outside the vocabulary (a prompt token, or a token chosen from
// logits without a finite value)?  The id was replaced by a valid one on the device, so nothing faulted, but the
// sequence's state is meaningless from there on: the sequence is closed until its next pacer_prefill.
int check_numeric(pacer_ctx* c, int s) {
  Seq& q = c->seq[s];
  if (!q.broken && !c->host_res[4 * PACER_MAX_BATCH + s]) return PACER_OK;
  q.pending = false;
  q.in_step = false;
  q.broken = true;
  return fail(c, PACER_ENUMERIC, "sequence %d: a token id outside the vocabulary was met (a prompt token out of range, or logits "
              "without a finite value); prefill the sequence again", s);
}

// M_B prefix rows (PosEmb row 0, K/V only) for positions no pre-verification call covered: the drafts beyond
// the last pre-verified block (bonus = false) or the position of the extra draft forward (bonus = true)
void mb_prefix_rows(pacer_ctx* c, const int* ids, int m, bool bonus) {
  SeqRows sr{};
  MbRows mr{};
  int R = 0, k = 0;
  for (int i = 0; i < m; ++i) {
    const Seq& q = c->seq[ids[i]];
    const int end = bonus ? q.verified + 1 : q.verified;       // draft positions [first, end)
    const int first = bonus ? q.verified : std::min(q.mb_done, q.verified);
    const int cnt = end - first;
    if (cnt <= 0) continue;
    sr.seq[k] = ids[i];
    sr.row_off[k] = R;
    sr.pos0[k] = q.len - 1 + first;
    sr.len[k] = q.len;
    mr.src_row0[k] = ids[i] * c->G1 + first;
    mr.e0[k] = -1;
    R += cnt;
    ++k;
  }
  sr.n_seqs = k;
  sr.row_off[k] = R;
  if (R > 0) run_preverify_rows(c, R, sr, mr, c->hidden, c->m[PACER_PREVERIFY].cfg.d_model, true);
}

// the acceptance kernels over `rows` rows per sequence (phase 0: rows i < gamma; phase 1: the bonus row)
void accept_launch(pacer_ctx* c, const AccArgs& aa, int rows, int phase, int mode, uint64_t seed, uint64_t ctr, const float* dev_logits,
                   int* dev_n, int* dev_z) {
  const int V = c->m[PACER_TARGET].cfg.vocab;
  if (rows > 0) {
    const dim3 grid(rows, aa.n_seqs, ACC_CHUNKS);
    if (mode != PACER_GREEDY)
      PACER_LAUNCH(accept_stats_kernel, grid, dim3(256), 0, c->stream, dev_logits, c->ring, aa, c->G1, V, phase, c->acc_part,
                   (const int*)nullptr);
    PACER_LAUNCH(accept_rows_kernel, grid, dim3(256), 0, c->stream, dev_logits, c->ring, c->draft_tok, aa, c->G1, V, mode, seed,
                 (uint32_t)ctr, phase, c->acc_part, c->rej, (const int*)nullptr);
  }
  PACER_LAUNCH(accept_finalize_kernel, dim3(aa.n_seqs), dim3(64), 0, c->stream, c->acc_part, c->rej, c->draft_tok, aa, c->G1, mode,
               phase, c->max_seq, c->tokens, dev_n, dev_z, c->host_res_dev, c->host_res_dev + 2 * PACER_MAX_BATCH, ++c->acc_calls, 0, V,
               host_bad_dev(c));
  for (int i = 0; i < aa.n_seqs; ++i) c->seq[aa.seq[i]].acc_ticket = c->acc_calls;
}

// Collects the results of every pending accept call.  A sequence whose phase 0 reports (gamma, -1) accepted every
// draft: its step still needs the draft forward on y_gamma (it completes the draft cache and yields the draft
// logits of the bonus row), M_B's prefix row for that position and the bonus row's token.  That part is
// enqueued here, once phase 0's result is known, for the sequences that need it, call by call.
int fold(pacer_ctx* c, int s) {
  if (!c->seq[s].pending) return PACER_OK;
  bool done[PACER_MAX_BATCH] = {false};
  for (int i = 0; i < c->max_batch; ++i) {
    Seq& o = c->seq[i];
    if (!o.pending || done[i]) continue;
    // the sequences of o's accept call carry the same ticket and were written by the same launch
    AccArgs ab{};
    int32_t sub[PACER_MAX_BATCH];
    int jb[PACER_MAX_BATCH];
    int m = 0;
    const int ticket = o.acc_ticket;
    for (int k = i; k < c->max_batch; ++k) {
      Seq& q = c->seq[k];
      if (!q.pending || q.acc_ticket != ticket) continue;
      done[k] = true;
      if (int rc = wait_ticket(c, c->host_res + 2 * PACER_MAX_BATCH + k, ticket, 0)) return rc;
      if (c->host_res[2 * k + 1] >= 0) continue;
      sub[m] = ab.seq[m] = ab.qslot[m] = k;
      jb[m] = q.verified;
      ab.slot[m] = q.acc_slot;
      ab.gamma[m] = q.verified;
      ab.len[m] = q.len;
      ab.beta[m] = q.acc_beta;
      ++m;
    }
    if (m > 0) {
      ab.n_seqs = m;
      draft_forward(c, sub, m, jb, PACER_GREEDY, 0, 0);
      mb_prefix_rows(c, sub, m, true);
      accept_launch(c, ab, 1, 1, o.acc_mode, o.acc_seed, o.acc_ctr, o.acc_logits, o.acc_n, o.acc_z);
      HIPCHK(c, hipGetLastError());
    }
  }
  for (int i = 0; i < c->max_batch; ++i) {
    Seq& o = c->seq[i];
    if (!o.pending) continue;
    if (int rc = wait_ticket(c, c->host_res + 2 * PACER_MAX_BATCH + i, o.acc_ticket, 0)) return rc;
    o.last_n = c->host_res[2 * i];
    o.last_z = c->host_res[2 * i + 1];
    o.len += o.last_n + 1;
    o.pending = false;
    if (c->host_res[4 * PACER_MAX_BATCH + i]) o.broken = true;   // reported by the sequence's own next call
  }
  return check_numeric(c, s);
}

// ---- acceptance without a context and without any allocation ---------------------------------
// The per-(row, vocabulary chunk) statistics and candidates and the per-row reject flags of the acceptance
// kernels, for PACER_NOALLOC_MAX_GAMMA + 1 rows, in an array that is part of the library's device image: each
// GPU the library runs on holds its own copy until the process ends.  Host code never uses the array's name as
// an address (on the host it is only a stand-in for the symbol): the device address is looked up once per
// device and kept.
constexpr int kNoAllocRows = PACER_NOALLOC_MAX_GAMMA + 1;
struct NoAllocScratch {
  float part[kNoAllocRows * ACC_CHUNKS * ACC_PART];
  int rej[kNoAllocRows];
};
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;
thread_local char g_err[256] = {0};     // last failure of a call that takes no context

int fail_noctx(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace

static __device__ __align__(256) unsigned char scratch[sizeof(NoAllocScratch)];

namespace {

// device address of `scratch` on the current device (looked up on the first call on that device)
int scratch_on_current_device(NoAllocScratch** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_noctx(PACER_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail_noctx(PACER_EHIP, "device index %d beyond the %d this library keeps scratch for", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail_noctx(PACER_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<NoAllocScratch*>(g_scratch_ptr[dev]);
  return PACER_OK;
}

}  // namespace

// =============================================================================================
extern "C" {

int32_t pacer_create(pacer_ctx** out, const pacer_model_cfg* target, const pacer_model_cfg* draft, const pacer_pv_cfg* pv,
                     int32_t max_batch, void* hip_stream) {
  if (!out || !target || !draft || !pv) return PACER_EINVAL;
  *out = nullptr;
  if (!cfg_ok(*target) || !cfg_ok(*draft)) return PACER_EINVAL;
  if (target->vocab != draft->vocab || target->max_seq != draft->max_seq) return PACER_EINVAL;
  if (pv->block < 1 || pv->gamma_max < pv->block || pv->gamma_max % pv->block || pv->gamma_max > 31) return PACER_EINVAL;
  if (!(pv->t0 >= 0.f) || !(pv->rho > 0.f)) return PACER_EINVAL;
  if (pv->halting < PACER_HALT_MEAN || pv->halting > PACER_HALT_LAST) return PACER_EINVAL;
  if (max_batch < 1 || max_batch > PACER_MAX_BATCH) return PACER_EINVAL;
  if (target->max_seq <= pv->gamma_max + 2) return PACER_EINVAL;
  pacer_ctx* c = new (std::nothrow) pacer_ctx();
  if (!c) return PACER_EINVAL;
  c->m[PACER_TARGET].cfg = *target;
  c->m[PACER_DRAFT].cfg = *draft;
  c->m[PACER_PREVERIFY].cfg = *draft;
  c->m[PACER_PREVERIFY].cfg.n_layers = 1;
  for (int w = 0; w < 3; ++w) {
    const int L = c->m[w].cfg.n_layers;
    c->m[w].attn_norm.assign(L, nullptr);
    c->m[w].ffn_norm.assign(L, nullptr);
    c->m[w].wqkv.assign(L, nullptr);
    c->m[w].wo.assign(L, nullptr);
    c->m[w].wgu.assign(L, nullptr);
    c->m[w].wd.assign(L, nullptr);
  }
  c->pv = *pv;
  c->max_batch = max_batch;
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->G1 = pv->gamma_max + 1;
  c->rcap = std::max(kPrefillRows, max_batch * c->G1);
  // attention partials: f32 models always go through them (all rows); bf16 models only when a decode
  // launch splits its keys, never in the wide prefill chunks
  c->prows = (target->dtype == PACER_F32 || draft->dtype == PACER_F32) ? c->rcap : std::max(kChunkRows, max_batch * c->G1);
  c->dmax = std::max(target->d_model, draft->d_model);
  c->fmax = std::max(target->d_ffn, draft->d_ffn);
  c->kmax = std::max(c->dmax, c->fmax);
  c->hmax = std::max(target->n_heads, draft->n_heads);
  c->hdmax = std::max(target->head_dim, draft->head_dim);
  c->max_seq = target->max_seq;
  c->lmax = std::max(target->n_layers, draft->n_layers);
  *out = c;
  return PACER_OK;
}

void pacer_destroy(pacer_ctx* c) {
  if (!c) return;
  if (c->ws_bound) {
    (void)hipStreamSynchronize(c->stream);
    for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    if (c->host_res) (void)hipHostFree(c->host_res);
  }
  delete c;
}

const char* pacer_last_error(const pacer_ctx* c) { return c ? c->err : (g_err[0] ? g_err : "null context"); }

int32_t pacer_pack_weight(void* dev_dst, const void* dev_src, int32_t n_out, int32_t n_in, int32_t tensor_id, int32_t head_dim,
                          int32_t* dev_not_finite, void* hip_stream) {
  if (!dev_dst || !dev_src || dev_dst == dev_src || n_out < 16 || n_in < 32 || n_out % 16 || n_in % 32) return PACER_EINVAL;
  int kind = PACK_PLAIN;
  if (tensor_id == PACER_T_WQKV) {
    if ((head_dim != 64 && head_dim != 128) || n_out % 3 || (n_out / 3) % head_dim) return PACER_EINVAL;
    kind = PACK_QKV;
  } else if (tensor_id == PACER_T_WGU) {
    if (n_out % 32) return PACER_EINVAL;
    kind = PACK_GATEUP;
  } else if (tensor_id != PACER_T_WO && tensor_id != PACER_T_WD && tensor_id != PACER_T_HEAD) {
    return PACER_EINVAL;
  }
  hipLaunchKernelGGL(pack_weight_kind_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(hip_stream), static_cast<uint4*>(dev_dst),
                     static_cast<const uint16_t*>(dev_src), n_out, n_in, kind, head_dim, dev_not_finite);
  return hipGetLastError() == hipSuccess ? PACER_OK : PACER_EHIP;
}

int32_t pacer_bind(pacer_ctx* c, int32_t which, int32_t tensor_id, int32_t layer, const void* p, uint64_t nbytes) {
  if (!c) return PACER_EINVAL;
  Model* m = model_of(c, which);
  if (!m || !p) return fail(c, PACER_EINVAL, "bind: bad model id or null pointer");
  const pacer_model_cfg& g = m->cfg;
  const uint64_t d = g.d_model, F = g.d_ffn, V = g.vocab, es = esize(g.dtype);
  const bool per_layer = tensor_id >= PACER_T_ATTN_NORM && tensor_id <= PACER_T_WD;
  if (per_layer && (layer < 0 || layer >= g.n_layers)) return fail(c, PACER_EINVAL, "bind: layer %d out of range", layer);
  uint64_t want = 0;
  switch (tensor_id) {
    case PACER_T_EMBED: want = V * d * es; break;
    case PACER_T_HEAD: want = V * d * es; break;
    case PACER_T_FINAL_NORM: case PACER_T_ATTN_NORM: case PACER_T_FFN_NORM: want = d * 4; break;
    case PACER_T_WQKV: want = 3 * d * d * es; break;
    case PACER_T_WO: want = d * d * es; break;
    case PACER_T_WGU: want = 2 * F * d * es; break;
    case PACER_T_WD: want = d * F * es; break;
    case PACER_T_POSEMB: want = (uint64_t)(c->pv.gamma_max + 1) * d * 4; break;
    case PACER_T_CLS: want = 2 * d * 4; break;
    default: return fail(c, PACER_EINVAL, "bind: unknown tensor id %d", tensor_id);
  }
  const bool mb_only = tensor_id == PACER_T_POSEMB || tensor_id == PACER_T_CLS;
  const bool lm_only = tensor_id == PACER_T_EMBED || tensor_id == PACER_T_HEAD;
  if ((mb_only && which != PACER_PREVERIFY) || (lm_only && which == PACER_PREVERIFY))
    return fail(c, PACER_EINVAL, "bind: tensor %d does not belong to model %d", tensor_id, which);
  if (nbytes != want) return fail(c, PACER_EINVAL, "bind: tensor %d expects %llu bytes, got %llu", tensor_id,
                                  (unsigned long long)want, (unsigned long long)nbytes);
  if (reinterpret_cast<uintptr_t>(p) % 16) return fail(c, PACER_EINVAL, "bind: pointer must be 16-byte aligned");
  switch (tensor_id) {
    case PACER_T_EMBED: m->embed = p; break;
    case PACER_T_HEAD: m->head = p; break;
    case PACER_T_FINAL_NORM: m->final_norm = static_cast<const float*>(p); break;
    case PACER_T_ATTN_NORM: m->attn_norm[layer] = static_cast<const float*>(p); break;
    case PACER_T_FFN_NORM: m->ffn_norm[layer] = static_cast<const float*>(p); break;
    case PACER_T_WQKV: m->wqkv[layer] = p; break;
    case PACER_T_WO: m->wo[layer] = p; break;
    case PACER_T_WGU: m->wgu[layer] = p; break;
    case PACER_T_WD: m->wd[layer] = p; break;
    case PACER_T_POSEMB: m->posemb = static_cast<const float*>(p); break;
    case PACER_T_CLS: m->cls = static_cast<const float*>(p); break;
  }
  return PACER_OK;
}

uint64_t pacer_kv_bytes(const pacer_ctx* c, int32_t which) {
  if (!c || which < 0 || which > 2) return 0;
  const pacer_model_cfg& g = c->m[which].cfg;
  return (uint64_t)c->max_batch * g.n_layers * 2 * g.max_seq * g.d_model * esize(g.dtype);
}

int32_t pacer_bind_kv(pacer_ctx* c, int32_t which, void* p, uint64_t nbytes) {
  if (!c) return PACER_EINVAL;
  if (which < 0 || which > 2 || !p) return fail(c, PACER_EINVAL, "bind_kv: bad model id or null pointer");
  if (nbytes != pacer_kv_bytes(c, which)) return fail(c, PACER_EINVAL, "bind_kv: expected %llu bytes",
                                                      (unsigned long long)pacer_kv_bytes(c, which));
  if (reinterpret_cast<uintptr_t>(p) % 16) return fail(c, PACER_EINVAL, "bind_kv: pointer must be 16-byte aligned");
  // attention reads whole 32-position groups; slots past a sequence's end must hold finite values
  HIPCHK(c, hipMemsetAsync(p, 0, nbytes, c->stream));
  c->m[which].kv = p;
  return PACER_OK;
}

uint64_t pacer_workspace_bytes(const pacer_ctx* c) {
  if (!c) return 0;
  pacer_ctx tmp = *c;   // carve on a copy with a null base only computes the size
  return carve(&tmp, nullptr);
}

int32_t pacer_bind_workspace(pacer_ctx* c, void* p, uint64_t nbytes) {
  if (!c) return PACER_EINVAL;
  if (!p || reinterpret_cast<uintptr_t>(p) % 256) return fail(c, PACER_EINVAL, "workspace must be non-null and 256-byte aligned");
  if (nbytes < pacer_workspace_bytes(c)) return fail(c, PACER_EINVAL, "workspace too small: need %llu bytes",
                                                     (unsigned long long)pacer_workspace_bytes(c));
  if (c->ws_bound) return fail(c, PACER_ESTATE, "workspace already bound");
  carve(c, p);
  HIPCHK(c, hipMemsetAsync(c->sk_cnt, 0, sizeof(unsigned) * kSplitGroups, c->stream));
  HIPCHK(c, hipMemsetAsync(c->att_cnt, 0, sizeof(unsigned) * PK_MAXB * c->hmax * 2, c->stream));
  for (int w = 0; w < 2; ++w)
    if (is_w16(c->m[w]))
      PACER_LAUNCH(rope_positions_kernel, dim3(c->max_seq), dim3(c->m[w].cfg.head_dim / 2), 0, c->stream, c->rope_pos[w], c->m[w].cfg.head_dim,
                   c->m[w].cfg.rope_theta);
  void* hp = nullptr;
  HIPCHK(c, hipHostMalloc(&hp, sizeof(int) * 5 * PACER_MAX_BATCH, hipHostMallocMapped));
  c->host_res = static_cast<int*>(hp);
  for (int i = 0; i < 5 * PACER_MAX_BATCH; ++i) c->host_res[i] = 0;
  void* dp = nullptr;
  HIPCHK(c, hipHostGetDevicePointer(&dp, hp, 0));
  c->host_res_dev = static_cast<int*>(dp);
  // attention keeps its 8 wave states in dynamic LDS: up to 8 x 32 rows x 132 floats = 132 KiB of the CU's 160
  {
    const int lds_max = 8 * 32 * (128 + 4) * 4;
#define PACER_ATT_LDS(HD_, MT_, QL_) HIPCHK(c, hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<HD_, MT_, QL_>), hipFuncAttributeMaxDynamicSharedMemorySize, lds_max))
    PACER_ATT_LDS(128, 2, 2); PACER_ATT_LDS(128, 1, 2); PACER_ATT_LDS(64, 2, 2); PACER_ATT_LDS(64, 1, 2);
    PACER_ATT_LDS(128, 2, 1); PACER_ATT_LDS(128, 1, 1); PACER_ATT_LDS(64, 2, 1); PACER_ATT_LDS(64, 1, 1);
#undef PACER_ATT_LDS
  }
  // the 8-wave wide GEMM stages its operand in dynamic LDS: up to 2 x 4 K steps x 6 row tiles x hi+lo KiB = 96 KiB
#define PACER_W8_LDS(HL_, MTB_, KSB_) HIPCHK(c, hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_wide8_kernel<EPI_RESID, 1, MTB_, HL_, 0, kWide8KC, KSB_>), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kWide8KC * MTB_ * HL_ * 1024))
  PACER_W8_LDS(2, 4, 2); PACER_W8_LDS(2, 4, 3); PACER_W8_LDS(2, 5, 2); PACER_W8_LDS(2, 5, 3); PACER_W8_LDS(2, 6, 2); PACER_W8_LDS(2, 6, 3);
#undef PACER_W8_LDS
#define PACER_W8_LDS(MTB_) HIPCHK(c, hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_wide8_kernel<EPI_SWIGLU, 2, MTB_, 2, 0, kWide8KC, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kWide8KC * MTB_ * 2 * 1024))
  PACER_W8_LDS(4); PACER_W8_LDS(5); PACER_W8_LDS(6);
#undef PACER_W8_LDS
  c->ws_bound = true;
  return PACER_OK;
}

int32_t pacer_prefill(pacer_ctx* c, int32_t s, const int32_t* dev_tokens, int32_t n) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (s < 0 || s >= c->max_batch || !dev_tokens || n < 1) return fail(c, PACER_EINVAL, "prefill: bad arguments");
  if (n + c->G1 + 1 > c->max_seq) return fail(c, PACER_EOVERFLOW, "prefill: %d tokens leave no room for a step (max_seq %d)", n, c->max_seq);
  Seq& q = c->seq[s];
  const bool q_was_used = q.len > 0;
  q = Seq();
  q.len = n;
  // a sequence that was in use may still have kernels in flight that report into its word: let them finish, then clear it
  if (q_was_used) HIPCHK(c, hipStreamSynchronize(c->stream));
  c->host_res[4 * PACER_MAX_BATCH + s] = 0;
  PACER_LAUNCH(copy_tokens_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, c->tokens + (size_t)s * c->max_seq, dev_tokens, n,
               c->m[PACER_TARGET].cfg.vocab, host_bad_dev(c), s);
  // up to 16 slots of 32 consecutive positions per pass: one trip through the weights per 512 prompt tokens
  for (int p0 = 0; p0 < n - 1; p0 += kPrefillRows) {
    const int R = std::min(kPrefillRows, n - 1 - p0);
    SeqRows sr{};
    MbRows mr{};
    sr.n_seqs = (R + kChunkRows - 1) / kChunkRows;
    for (int i = 0; i < sr.n_seqs; ++i) {
      sr.seq[i] = s;
      sr.row_off[i] = i * kChunkRows;
      sr.pos0[i] = p0 + i * kChunkRows;
      sr.len[i] = n;
      mr.src_row0[i] = i * kChunkRows;
      mr.e0[i] = -1;
    }
    sr.row_off[sr.n_seqs] = R;
    forward_lm(c, c->m[PACER_TARGET], 0, R, sr, true);       // the target's prompt pass leaves nothing but its cache rows
    const Model& md = c->m[PACER_DRAFT];
    forward_lm(c, md, 1, R, sr);
    // the draft's hidden states (final-norm output) feed M_B's prefix rows; staged in ao
    if (is_w16(md))
      PACER_LAUNCH(hidden_rows_kernel, dim3(R), dim3(256), 0, c->stream, c->x, c->dmax, md.final_norm, slot(c, 2 * md.cfg.n_layers),
                         c->rcap, 1.0f / md.cfg.d_model, md.cfg.rms_eps, md.cfg.d_model, c->ao, c->dmax);
    else
      (void)hipMemcpy2DAsync(c->ao, (size_t)c->dmax * 4, c->xn, (size_t)c->kmax * 4, (size_t)md.cfg.d_model * 4, R, hipMemcpyDeviceToDevice,
                             c->stream);
    run_preverify_rows(c, R, sr, mr, c->ao, c->dmax, true);
  }
  HIPCHK(c, hipGetLastError());
  return PACER_OK;
}

int32_t pacer_force_commit(pacer_ctx* c, int32_t s, int32_t from, const int32_t* host_tokens, int32_t n) {
  if (!c) return PACER_EINVAL;
  if (!c->ws_bound) return fail(c, PACER_ESTATE, "workspace not bound");
  if (s < 0 || s >= c->max_batch || !host_tokens || n < 1 || from < 0) return fail(c, PACER_EINVAL, "force_commit: bad arguments");
  if (from + n + c->G1 + 1 > c->max_seq) return fail(c, PACER_EOVERFLOW, "force_commit: beyond max_seq");
  for (int i = 0; i < n; ++i)
    if (host_tokens[i] < 0 || host_tokens[i] >= c->m[PACER_TARGET].cfg.vocab)
      return fail(c, PACER_EINVAL, "force_commit: token %d (index %d) is outside the vocabulary", host_tokens[i], i);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(c->tokens + (size_t)s * c->max_seq + from, host_tokens, sizeof(int) * n, hipMemcpyHostToDevice));
  Seq& q = c->seq[s];
  q.pending = false;
  q.in_step = false;
  c->pre_valid = false;
  q.len = from + n;
  q.gamma = q.mb_done = 0;
  q.verified = -1;
  return PACER_OK;
}

int32_t pacer_begin_step(pacer_ctx* c, int32_t s) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (s < 0 || s >= c->max_batch) return fail(c, PACER_EINVAL, "begin_step: sequence id %d out of range", s);
  if (c->hip_failed) {
    // the cross-block hand-overs rely on their arrival counters being zero between launches
    c->hip_failed = false;
    HIPCHK(c, hipMemsetAsync(c->sk_cnt, 0, sizeof(unsigned) * kSplitGroups, c->stream));
    HIPCHK(c, hipMemsetAsync(c->att_cnt, 0, sizeof(unsigned) * PK_MAXB * c->hmax * 2, c->stream));
  }
  if (int rc = fold(c, s)) return rc;
  if (int rc = check_numeric(c, s)) return rc;
  Seq& q = c->seq[s];
  if (q.len < 1) return fail(c, PACER_ESTATE, "begin_step: sequence %d has no committed tokens (prefill first)", s);
  if (q.len + c->G1 + 1 > c->max_seq) return fail(c, PACER_EOVERFLOW, "begin_step: sequence %d is full", s);
  q.t = c->pv.t0;
  q.gamma = q.mb_done = 0;
  q.verified = -1;
  q.in_step = true;
  c->pre_valid = false;
  return PACER_OK;
}

int32_t pacer_draft_step(pacer_ctx* c, const int32_t* seqs, int32_t n, int32_t mode, uint64_t seed, uint64_t ctr) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (int rc = check_seqs(c, seqs, n)) return rc;
  if (mode != PACER_GREEDY && mode != PACER_SAMPLE) return fail(c, PACER_EINVAL, "draft_step: bad mode %d", mode);
  int j[PACER_MAX_BATCH];
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    if (!q.in_step || q.verified >= 0) return fail(c, PACER_ESTATE, "draft_step: sequence %d is not drafting (begin_step first)", seqs[i]);
    if (q.gamma >= c->pv.gamma_max) return fail(c, PACER_EOVERFLOW, "draft_step: sequence %d already holds gamma_max drafts", seqs[i]);
    j[i] = q.gamma;
  }
  draft_forward(c, seqs, n, j, mode, seed, ctr);
  for (int i = 0; i < n; ++i) c->seq[seqs[i]].gamma++;
  HIPCHK(c, hipGetLastError());
  return PACER_OK;
}

int32_t pacer_preverify_block(pacer_ctx* c, const int32_t* seqs, int32_t n, float* dev_alpha, int32_t* dev_stop) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (int rc = check_seqs(c, seqs, n)) return rc;
  if (!dev_alpha || !dev_stop) return fail(c, PACER_EINVAL, "preverify_block: null output");
  const int b = c->pv.block;
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    if (!q.in_step || q.verified >= 0 || q.gamma - q.mb_done != b)
      return fail(c, PACER_ESTATE, "preverify_block: sequence %d needs exactly %d new drafts", seqs[i], b);
  }
  SeqRows sr{};
  MbRows mr{};
  HaltArgs ha{};
  sr.n_seqs = ha.n_seqs = n;
  ha.rule = c->pv.halting;
  for (int i = 0; i < n; ++i) {
    Seq& q = c->seq[seqs[i]];
    sr.seq[i] = seqs[i];
    sr.row_off[i] = i * b;
    sr.pos0[i] = q.len - 1 + q.mb_done;
    sr.len[i] = q.len;
    mr.src_row0[i] = seqs[i] * c->G1 + q.mb_done;
    mr.e0[i] = q.mb_done + 1;                 // draft positions i, i+1, ... (1-based)
    ha.t[i] = q.t;
    ha.seq[i] = seqs[i];
    ha.ticket[i] = q.pv_ticket = c->pv_calls + 1;   // per context, never reused: a re-prefilled sequence cannot match a stale word
    ha.force[i] = q.force;
    q.force = -1;
  }
  ++c->pv_calls;
  sr.row_off[n] = n * b;
  const Model& mb = c->m[PACER_PREVERIFY];
  run_preverify_rows(c, n * b, sr, mr, c->hidden, mb.cfg.d_model, false);
  // one sequence, bf16 models: the head kernel goes on to embed the newest draft token, which is what the next
  // round's first draft step starts with if drafting goes on (if it stops, the verify pass overwrites it)
  const Seq& q0 = c->seq[seqs[0]];
  const bool embed_next = n == 1 && is_w16(mb) && is_w16(c->m[PACER_DRAFT]) && q0.gamma < c->pv.gamma_max;
  preverify_head(c, n, b, ha, dev_alpha, dev_stop, embed_next ? c->draft_tok + seqs[0] * c->G1 + (q0.gamma - 1) : nullptr);
  if (embed_next) {
    c->pre_valid = true;
    c->pre_n = 1;
    c->pre_seq[0] = seqs[0];
    c->pre_j[0] = q0.gamma;
  }
  for (int i = 0; i < n; ++i) {
    Seq& q = c->seq[seqs[i]];
    q.mb_done += b;
    q.t = q.t * c->pv.rho;
  }
  HIPCHK(c, hipGetLastError());
  return PACER_OK;
}

int32_t pacer_force_stop(pacer_ctx* c, int32_t s, int32_t flag) {
  if (!c) return PACER_EINVAL;
  if (s < 0 || s >= c->max_batch) return fail(c, PACER_EINVAL, "force_stop: sequence id %d out of range", s);
  if (flag < -1 || flag > 1) return fail(c, PACER_EINVAL, "force_stop: flag must be -1, 0 or 1");
  c->seq[s].force = flag;
  return PACER_OK;
}

int32_t pacer_wait_stop(pacer_ctx* c, const int32_t* seqs, int32_t n, int32_t* host_stop) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (int rc = check_seqs(c, seqs, n)) return rc;
  if (!host_stop) return fail(c, PACER_EINVAL, "wait_stop: null output");
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    if (q.pv_ticket == 0) return fail(c, PACER_ESTATE, "wait_stop: sequence %d has had no pre-verification call", seqs[i]);
    const int* p = c->host_res + 3 * PACER_MAX_BATCH + seqs[i];
    if (int rc = wait_ticket(c, p, q.pv_ticket, 1)) return rc;
    host_stop[i] = *p & 1;
  }
  for (int i = 0; i < n; ++i)
    if (int rc = check_numeric(c, seqs[i])) return rc;
  return PACER_OK;
}

int32_t pacer_draft_window(pacer_ctx* c, const int32_t* seqs, int32_t n, int32_t mode, uint64_t seed, uint64_t ctr, float* dev_alpha,
                           int32_t* dev_stop, int32_t* host_gamma) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (int rc = check_seqs(c, seqs, n)) return rc;
  if (!dev_alpha || !dev_stop || !host_gamma) return fail(c, PACER_EINVAL, "draft_window: null output");
  if (mode != PACER_GREEDY && mode != PACER_SAMPLE) return fail(c, PACER_EINVAL, "draft_window: bad mode %d", mode);
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    if (!q.in_step || q.verified >= 0 || q.gamma != 0) return fail(c, PACER_ESTATE, "draft_window: sequence %d is not at the start of a step", seqs[i]);
  }
  // the inner loop of Alg. 1: blocks of b draft steps and one pre-verification call for the sequences still drafting
  int32_t active[PACER_MAX_BATCH], flags[PACER_MAX_BATCH];
  int m = n;
  for (int i = 0; i < n; ++i) active[i] = seqs[i];
  const int b = c->pv.block;
  while (m > 0) {
    for (int k = 0; k < b; ++k)
      if (int rc = pacer_draft_step(c, active, m, mode, seed, ctr)) return rc;
    if (int rc = pacer_preverify_block(c, active, m, dev_alpha, dev_stop)) return rc;
    if (int rc = pacer_wait_stop(c, active, m, flags)) return rc;
    int keep = 0;
    for (int i = 0; i < m; ++i)
      if (!flags[i] && c->seq[active[i]].gamma + b <= c->pv.gamma_max) active[keep++] = active[i];
    m = keep;
  }
  for (int i = 0; i < n; ++i) host_gamma[i] = c->seq[seqs[i]].gamma;
  return PACER_OK;
}

int32_t pacer_verify(pacer_ctx* c, const int32_t* seqs, int32_t n, const int32_t* gamma_override, float* dev_logits) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (int rc = check_seqs(c, seqs, n)) return rc;
  if (!dev_logits) return fail(c, PACER_EINVAL, "verify: null output");
  int g[PACER_MAX_BATCH];
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    if (!q.in_step) return fail(c, PACER_ESTATE, "verify: sequence %d has no step in progress", seqs[i]);
    g[i] = (gamma_override && gamma_override[i] >= 0) ? gamma_override[i] : q.gamma;
    if (g[i] > q.gamma) return fail(c, PACER_EINVAL, "verify: gamma %d exceeds the %d drafts made", g[i], q.gamma);
  }
  SeqRows sr{};
  sr.n_seqs = n;
  int R = 0;
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    sr.seq[i] = seqs[i];
    sr.row_off[i] = R;
    sr.pos0[i] = q.len - 1;
    sr.len[i] = q.len;
    R += g[i] + 1;
  }
  sr.row_off[n] = R;
  const Model& mt = c->m[PACER_TARGET];
  forward_lm(c, mt, 0, R, sr);
  lm_head(c, mt, 0, R, dev_logits, sr, ROWMAP_LIST);
  for (int i = 0; i < n; ++i) c->seq[seqs[i]].verified = g[i];
  HIPCHK(c, hipGetLastError());
  return PACER_OK;
}

int32_t pacer_accept_rollback(pacer_ctx* c, const int32_t* seqs, int32_t n, int32_t mode, const float* beta, uint64_t seed,
                              uint64_t ctr, const float* dev_logits, int32_t* dev_n, int32_t* dev_z) {
  if (!c) return PACER_EINVAL;
  if (int rc = ready(c)) return rc;
  if (int rc = check_seqs(c, seqs, n)) return rc;
  if (!beta || !dev_logits || !dev_n || !dev_z) return fail(c, PACER_EINVAL, "accept_rollback: null argument");
  if (mode != PACER_GREEDY && mode != PACER_SAMPLE) return fail(c, PACER_EINVAL, "accept_rollback: bad mode %d", mode);
  for (int i = 0; i < n; ++i)
    if (!c->seq[seqs[i]].in_step || c->seq[seqs[i]].verified < 0)
      return fail(c, PACER_ESTATE, "accept_rollback: sequence %d has not been verified", seqs[i]);
  // Rows i < gamma only: M_B prefix rows for the drafts no pre-verification call covered, the accept tests and
  // the token at the first rejection.  The bonus row (needed only by a sequence that accepted every draft, and
  // costing one more draft forward) is enqueued by whichever call collects the result (see fold), so this call
  // returns without waiting for the verify pass.
  for (int i = 0; i < n; ++i)
    if (c->seq[seqs[i]].pending) return fail(c, PACER_ESTATE, "accept_rollback: sequence %d has an uncollected result", seqs[i]);
  mb_prefix_rows(c, seqs, n, false);
  AccArgs aa{};
  aa.n_seqs = n;
  int gmax = 0;
  for (int i = 0; i < n; ++i) {
    const Seq& q = c->seq[seqs[i]];
    aa.seq[i] = aa.qslot[i] = seqs[i];
    aa.slot[i] = i;
    aa.gamma[i] = q.verified;
    aa.len[i] = q.len;
    aa.beta[i] = beta[i];
    gmax = std::max(gmax, q.verified);
  }
  accept_launch(c, aa, gmax, 0, mode, seed, ctr, dev_logits, dev_n, dev_z);
  for (int i = 0; i < n; ++i) {
    Seq& q = c->seq[seqs[i]];
    q.pending = true;
    q.in_step = false;
    q.acc_mode = mode; q.acc_slot = i; q.acc_beta = beta[i]; q.acc_seed = seed; q.acc_ctr = ctr;
    q.acc_logits = dev_logits; q.acc_n = dev_n; q.acc_z = dev_z;
  }
  HIPCHK(c, hipGetLastError());
  return PACER_OK;
}

int32_t pacer_accept_noalloc(const float* dev_target_logits, const float* dev_draft_logits, const int32_t* dev_draft_tokens,
                             int32_t gamma, int32_t bonus_row, int32_t vocab, int32_t mode, float beta, uint64_t seed, uint64_t ctr,
                             int32_t seq, int32_t* dev_n, int32_t* dev_z, void* hip_stream) {
  if (!dev_target_logits || !dev_draft_logits || !dev_draft_tokens || !dev_n || !dev_z)
    return fail_noctx(PACER_EINVAL, "accept_noalloc: null argument");
  if (gamma < 0 || vocab < 1 || seq < 0 || seq >= PACER_MAX_BATCH) return fail_noctx(PACER_EINVAL, "accept_noalloc: bad gamma, vocab or sequence id");
  if (mode != PACER_GREEDY && mode != PACER_SAMPLE) return fail_noctx(PACER_EINVAL, "accept_noalloc: bad mode %d", mode);
  if (gamma > PACER_NOALLOC_MAX_GAMMA)
    return fail_noctx(PACER_EOVERFLOW, "accept_noalloc: gamma %d exceeds PACER_NOALLOC_MAX_GAMMA = %d (the fixed scratch holds %d rows)", gamma,
                      PACER_NOALLOC_MAX_GAMMA, kNoAllocRows);
  if (gamma == 0 && !bonus_row) return fail_noctx(PACER_EINVAL, "accept_noalloc: nothing to evaluate (gamma 0 and no bonus row)");
  NoAllocScratch* sc = nullptr;
  if (int rc = scratch_on_current_device(&sc)) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  AccArgs aa{};
  aa.n_seqs = 1;
  aa.seq[0] = seq;
  aa.slot[0] = 0;
  aa.qslot[0] = 0;
  aa.gamma[0] = gamma;
  aa.len[0] = 0;
  aa.beta[0] = beta;
  const int G1 = gamma + 1;
  // Every word of the scratch that a launch reads was written earlier in this same call (statistics by
  // accept_stats, candidates and reject flags by accept_rows), so nothing has to start at zero.
  for (int phase = 0; phase < (bonus_row ? 2 : 1); ++phase) {
    const int rows = phase ? 1 : gamma;
    if (rows > 0) {
      const dim3 grid(rows, 1, ACC_CHUNKS);
      const int* done = phase ? dev_z : nullptr;
      if (mode != PACER_GREEDY)
        hipLaunchKernelGGL(accept_stats_kernel, grid, dim3(256), 0, st, dev_target_logits, dev_draft_logits, aa, G1, vocab, phase, sc->part, done);
      hipLaunchKernelGGL(accept_rows_kernel, grid, dim3(256), 0, st, dev_target_logits, dev_draft_logits, dev_draft_tokens, aa, G1, vocab, mode,
                         seed, (uint32_t)ctr, phase, sc->part, sc->rej, done);
    }
    hipLaunchKernelGGL(accept_finalize_kernel, dim3(1), dim3(64), 0, st, sc->part, sc->rej, dev_draft_tokens, aa, G1, mode, phase, 0,
                       (int*)nullptr, dev_n, dev_z, (int*)nullptr, (int*)nullptr, 0, 1, vocab, (int*)nullptr);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_noctx(PACER_EHIP, "accept_noalloc: %s", hipGetErrorString(e));
  return PACER_OK;
}

int32_t pacer_get_state(pacer_ctx* c, int32_t s, int32_t* gamma, int32_t* len, float* t, int32_t* n_acc, int32_t* next) {
  if (!c) return PACER_EINVAL;
  if (s < 0 || s >= c->max_batch) return fail(c, PACER_EINVAL, "get_state: sequence id %d out of range", s);
  if (c->ws_bound) {
    if (int rc = fold(c, s)) return rc;
    if (int rc = check_numeric(c, s)) return rc;
  }
  const Seq& q = c->seq[s];
  if (gamma) *gamma = q.gamma;
  if (len) *len = q.len;
  if (t) *t = q.t;
  if (n_acc) *n_acc = q.last_n;
  if (next) *next = q.last_z;
  return PACER_OK;
}

int32_t pacer_peek(pacer_ctx* c, int32_t s, int32_t what, void** p, uint64_t* nbytes) {
  if (!c) return PACER_EINVAL;
  if (!c->ws_bound) return fail(c, PACER_ESTATE, "workspace not bound");
  if (s < 0 || s >= c->max_batch || !p || !nbytes) return fail(c, PACER_EINVAL, "peek: bad arguments");
  const int V = c->m[PACER_DRAFT].cfg.vocab, dD = c->m[PACER_DRAFT].cfg.d_model, G1 = c->G1;
  switch (what) {
    case PACER_PEEK_DRAFT_LOGITS: *p = c->ring + (size_t)s * G1 * V; *nbytes = (uint64_t)G1 * V * 4; break;
    case PACER_PEEK_DRAFT_HIDDEN: *p = c->hidden + (size_t)s * G1 * dD; *nbytes = (uint64_t)G1 * dD * 4; break;
    case PACER_PEEK_DRAFT_TOKENS: *p = c->draft_tok + s * G1; *nbytes = (uint64_t)G1 * 4; break;
    case PACER_PEEK_TOKENS: *p = c->tokens + (size_t)s * c->max_seq; *nbytes = (uint64_t)c->max_seq * 4; break;
    default: return fail(c, PACER_EINVAL, "peek: unknown buffer %d", what);
  }
  return PACER_OK;
}

int32_t pacer_launch_plan(int32_t n_out, int32_t n_in, int32_t rows, int32_t operand_parts, int32_t* tiles_per_block,
                          int32_t* k_slices) {
  if (!tiles_per_block || !k_slices || n_out < 16 || n_out % 16 || n_out / 16 >= 512 || n_in < 32 || n_in % 32 || rows < 1 ||
      rows > 32 || operand_parts < 1 || operand_parts > 2)
    return PACER_EINVAL;
  const SplitShape sp = n_in / 32 >= 64 ? pick_split_shape(n_out / 16, n_in / 32, rows, operand_parts) : SplitShape{1, 1};
  *tiles_per_block = sp.nt;
  *k_slices = sp.ksb;
  return PACER_OK;
}

int32_t pacer_launch_count(const pacer_ctx* c, int64_t* n_launches) {
  if (!c || !n_launches) return PACER_EINVAL;
  *n_launches = c->n_launches;
  return PACER_OK;
}

int32_t pacer_stream_probe(const void* dev_src, uint64_t nbytes, int32_t repeat, void* dev_sink, void* hip_stream) {
  if (!dev_src || !dev_sink || nbytes < 16 || repeat < 1 || repeat > 100000 || reinterpret_cast<uintptr_t>(dev_src) % 16)
    return fail_noctx(PACER_EINVAL, "stream_probe: bad arguments");
  for (int r = 0; r < repeat; ++r)
    hipLaunchKernelGGL(stream_probe_kernel, dim3(256), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4*>(dev_src), (size_t)(nbytes / 16), static_cast<uint32_t*>(dev_sink));
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_noctx(PACER_EHIP, "stream_probe: %s", hipGetErrorString(e));
  return PACER_OK;
}

int32_t pacer_profile_enable(pacer_ctx* c, int32_t on) {
  if (!c) return PACER_EINVAL;
  if (!c->ws_bound) return fail(c, PACER_ESTATE, "workspace not bound");
  if (on && c->ev.empty()) {
    c->ev.resize(kProfEvents);
    for (auto& e : c->ev) HIPCHK(c, hipEventCreate(&e));
  }
  c->prof = on != 0;
  return PACER_OK;
}

int32_t pacer_profile_read(pacer_ctx* c, int64_t* n_launches, double* total_ms, double* weight_bytes) {
  if (!c) return PACER_EINVAL;
  if (!c->ws_bound) return fail(c, PACER_ESTATE, "workspace not bound");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  double ms = 0.0;
  for (int i = 0; i + 1 < c->n_ev; i += 2) {
    float t = 0.f;
    HIPCHK(c, hipEventElapsedTime(&t, c->ev[i], c->ev[i + 1]));
    ms += t;
  }
  if (n_launches) *n_launches = c->n_ev / 2;
  if (total_ms) *total_ms = ms;
  if (weight_bytes) *weight_bytes = c->prof_bytes;
  c->n_ev = 0;
  c->prof_bytes = 0.0;
  return PACER_OK;
}

}  // extern "C"
