// Fused kernels of the bf16-weight path (gfx950, wave64, v_mfma_f32_16x16x32_f16).
//
// One decoder layer is five launches:
//   QKV GEMM   (epilogue: row scale of the RMSNorm, RoPE, Q -> f16 attention operand, K/V -> cache)
//   attention  (MFMA scores and weighted values, 8 waves per key range merged through LDS, output = the
//               f16 operand of the O projection; few heads or long contexts: several key ranges per
//               head, combined by the block that finishes last)
//   O GEMM     (epilogue: residual add, next norm's operand x*g as f16, row sum of squares)
//   gate/up GEMM (epilogue: row scale, SwiGLU, f16 operand of the down projection)
//   down GEMM  (epilogue: residual add, next norm's operand, row sum of squares)
//
// RMSNorm never runs as a kernel: x*g is what the consuming GEMM multiplies, and the per-row factor
// 1/sqrt(mean x^2 + eps) commutes with the matrix product, so it is applied to the accumulators.  The
// row sums of squares are accumulated by the producing GEMM's blocks with integer (fixed point,
// 2^-26) atomics: integer addition is associative, so the result does not depend on block order.
//
// Weight tiles hold the bf16 values converted to f16 (see kernels.h).  Tile layouts (written by pack_weight_kind_kernel):
//   PLAIN   tile nt, row i  <- matrix row 16*nt + i
//   QKV     Q and K parts: a tile holds 8 rotation pairs of one head: row i<8 <- dim 8t+i, row i+8 <-
//           dim 8t+i+hd/2 (t = tile within the head); V part plain.  RoPE then stays inside a tile.
//   GATEUP  tile nt: rows 0..7 <- gate rows 8nt..8nt+7, rows 8..15 <- up rows 8nt..8nt+7.
// KV cache of a bf16 model, per (sequence, layer): K then V, both f16, both stored per head in the
// order the attention MFMAs read them, so that every operand load of a wave is one contiguous 1 KiB:
//   K  [head][position/16][feature/32][lane][8]   lane = 16*((feature%32)/8) + position%16
//   V  [head][position/32][feature/16][lane][8]   lane = 16*((position%16)/4) + feature%16,
//                                                 element = position%4 + 4*((position%32)/16)
// (A row-major [position][d] cache makes a wave's 16 rows of one load sit a power of two apart, which
// serialises them on one memory channel: measured 4x slower at 550 keys.)
#pragma once
#include "kernels.h"

// The cross-block hand-overs below rest on gfx950 behaviour (see "KSB" at gemm_w16_kernel) and on the encoding of
// s_waitcnt for that target: refuse to build device code for anything else.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "kernels_w16.h is written for gfx950 (MI355X): the fence-free hand-over and the s_waitcnt immediates are specific to it"
#endif
// Memory order of the arrival-counter increment of those hand-overs.  Relaxed by default: ordering comes from the
// write-through stores having completed (vmcnt 0) before the block's barrier, and from loads that do not hit in L2.
// Building with -DPACER_FENCED_HANDOVER makes the increment an agent-scope acquire-release (L2 write-back before it,
// invalidation after it, 4 to 15 us per launch): the variant to compare with if results ever differ between runs.
#ifdef PACER_FENCED_HANDOVER
#define PACER_HO_ORDER __ATOMIC_ACQ_REL
#else
#define PACER_HO_ORDER __ATOMIC_RELAXED
#endif
#define PACER_WAIT_VMCNT0() __builtin_amdgcn_s_waitcnt(0x0F70)   // gfx9 encoding: vmcnt = 0, expcnt and lgkmcnt at their maxima (no wait)

#define PACK_PLAIN 0
#define PACK_QKV 1
#define PACK_GATEUP 2

#define EPI_STORE 0
#define EPI_RESID 1
#define EPI_QKV 2
#define EPI_SWIGLU 3

#define SSQ_SCALE 67108864.0f            // 2^26
#define SSQ_INV_SCALE 1.4901161193847656e-08f

typedef unsigned long long u64;

// A slot of row sums is SSQ_SUB interleaved accumulators [sub][stride] (blocks spread their atomics
// over them to cut contention); the sum of the parts is an integer sum, so still order independent.
#define SSQ_SUB 8
__device__ __forceinline__ float row_scale(const u64* ssq, int stride, int m, float inv_dim, float eps) {
  u64 t = 0;
#pragma unroll
  for (int i = 0; i < SSQ_SUB; ++i) t += ssq[(size_t)i * stride + m];
  return 1.0f / sqrtf((float)t * SSQ_INV_SCALE * inv_dim + eps);
}
// row r's accumulators of every slot: slot 0 part 0 = v, everything else 0
__device__ __forceinline__ void ssq_init_row(u64* ssq, int n_slots, int stride, int r, float ss) {
  for (int i = threadIdx.x; i < n_slots * SSQ_SUB; i += blockDim.x) ssq[(size_t)i * stride + r] = (i == 0) ? (u64)(ss * SSQ_SCALE + 0.5f) : 0ull;
}

// bad (may be null): incremented once per weight whose half-float value is not finite (|w| > 65504, inf, NaN)
__global__ void pack_weight_kind_kernel(uint4* __restrict__ dst, const uint16_t* __restrict__ src, int N, int K, int kind, int param,
                                        int* __restrict__ bad) {
  const int KT = K >> 5;
  const size_t total = (size_t)(N >> 4) * KT * 64;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = (int)(idx & 63);
    const size_t tile = idx >> 6;
    const int kt = (int)(tile % KT);
    const int nt = (int)(tile / KT);
    const int i = lane & 15;
    int row = nt * 16 + i;
    if (kind == PACK_QKV) {
      const int hd = param, d = N / 3;
      if (row < 2 * d) {
        const int part = (nt * 16) / d;                 // 0 = Q, 1 = K
        const int tq = nt - part * (d / 16);            // tile within the part
        const int tph = hd / 16;                        // tiles per head
        const int h = tq / tph, t = tq % tph;
        row = part * d + h * hd + 8 * t + (i & 7) + (i >> 3) * (hd / 2);
      }
    } else if (kind == PACK_GATEUP) {
      const int F = N / 2;
      row = (i < 8) ? (8 * nt + i) : (F + 8 * nt + (i - 8));
    }
    const uint16_t* p = src + (size_t)row * K + kt * 32 + (lane >> 4) * 8;
    const u32x4 h = bf16x8_to_f16x8(*reinterpret_cast<const u32x4*>(p));
    dst[idx] = make_uint4(h[0], h[1], h[2], h[3]);
    if (bad) {
      int nb = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) nb += ((h[e] & 0x7c00u) == 0x7c00u) + ((h[e] & 0x7c000000u) == 0x7c000000u);   // exponent all ones
      if (nb) atomicAdd(bad, nb);
    }
  }
}

// ------------------------------------------------------------------ producers of layer-0 input
// The f16 operand of a GEMM is stored as two tiles per (k tile, row tile): hi = f16(v) and
// lo = f16(v - hi).  hi alone carries 11 significant bits; 32 layers of a 4096-wide model turn that
// rounding into 1.5e-2 of the logit RMS (measured against the float64 oracle and reproduced by rounding
// the oracle's activations), so the target model's GEMMs multiply both tiles into the same accumulator.
// Layout: [k tile][row tile][hi|lo][row in tile][32 features]: inside a 1 KiB tile a row is 64
// contiguous bytes, and MFMA lane 16*g + j reads bytes 64*j + 16*g..+15 of it.  (Storing the tile in
// lane order instead makes a launch with 9..16 rows touch all eight 128-byte lines of every tile and
// measured 5 to 10 % slower GEMMs; this way the lines touched follow the row count.)
// 4 consecutive features of row m into the packed operand
__device__ __forceinline__ void store_packed4(_Float16* __restrict__ xp, int MT_total, int m, int k0, float a, float b, float c, float d) {
  const int kt = k0 >> 5, g = (k0 & 31) >> 3, e = k0 & 7;
  typedef _Float16 half4 __attribute__((ext_vector_type(4)));
  const half4 h = {(_Float16)a, (_Float16)b, (_Float16)c, (_Float16)d};
  const half4 l = {(_Float16)(a - (float)h[0]), (_Float16)(b - (float)h[1]), (_Float16)(c - (float)h[2]), (_Float16)(d - (float)h[3])};
  _Float16* p = xp + ((size_t)(kt * MT_total + (m >> 4)) * 128 + ((m & 15) * 4 + g)) * 8 + e;
  *reinterpret_cast<half4*>(p) = h;
  *reinterpret_cast<half4*>(p + 512) = l;
}

// x = E[token]; operand = f16(x * g); ssq slot 0 = sum x^2; the row's accumulators of the other slots are cleared.
// cos/sin of every absolute position for a model's rotation frequencies, evaluated in double and rounded once:
// tab[pos][j] = (cos, sin)(pos * theta^(-2j/hd)).  Filled when the workspace is bound; the QKV epilogue reads the
// row of a token's position.  grid = max_seq, block = hd/2
__global__ void rope_positions_kernel(float* __restrict__ tab, int hd, float theta) {
  const int pos = blockIdx.x, j = threadIdx.x, half = hd >> 1;
  if (j >= half) return;
  const double inv = pow((double)theta, -2.0 * (double)j / (double)hd);
  double sn, cs;
  sincos((double)pos * inv, &sn, &cs);
  tab[((size_t)pos * half + j) * 2] = (float)cs;
  tab[((size_t)pos * half + j) * 2 + 1] = (float)sn;
}

// Row r of a forward's input from embedding row e: x, the first norm's operand f16(x * g) and the row's sums of
// squares (slot 0 = sum x^2, the other slots cleared).  Called by all threads of a block.
struct EmbedOut {
  float* x;              // residual stream rows [.][ldx]
  int ldx;
  const float* g;        // gain of the first layer's attention norm
  _Float16* xp;          // operand of the first GEMM
  int MT_total;
  u64* ssq;
  int n_slots, slot_stride;
};
__device__ __forceinline__ void embed_row_w16(const uint16_t* __restrict__ e, int d, int r, const EmbedOut& o, float* red) {
  uint2 w0 = {0u, 0u};
  if ((int)threadIdx.x * 4 < d) w0 = *reinterpret_cast<const uint2*>(e + threadIdx.x * 4);
  float ss = 0.f;
  for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
    const uint2 w = k == (int)threadIdx.x * 4 ? w0 : *reinterpret_cast<const uint2*>(e + k);
    const float v0 = __uint_as_float(w.x << 16), v1 = __uint_as_float(w.x & 0xffff0000u);
    const float v2 = __uint_as_float(w.y << 16), v3 = __uint_as_float(w.y & 0xffff0000u);
    *reinterpret_cast<float4*>(o.x + (size_t)r * o.ldx + k) = make_float4(v0, v1, v2, v3);
    store_packed4(o.xp, o.MT_total, r, k, v0 * o.g[k], v1 * o.g[k + 1], v2 * o.g[k + 2], v3 * o.g[k + 3]);
    ss += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3;
  }
  ss = block_sum(ss, red);
  ssq_init_row(o.ssq, o.n_slots, o.slot_stride, r, ss);
}

__global__ void embed_w16_kernel(const uint16_t* __restrict__ E, const int* __restrict__ tokens, const int* __restrict__ draft_tok,
                                 SeqRows sr, int max_seq, int G1, int d, EmbedOut out) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  const int si = find_seq(sr, r);
  const int s = sr.seq[si];
  const int p = sr.pos0[si] + (r - sr.row_off[si]);
  const int tok = p < sr.len[si] ? tokens[(size_t)s * max_seq + p] : draft_tok[s * G1 + (p - sr.len[si])];
  embed_row_w16(E + (size_t)tok * d, d, r, out, red);
}

// input rows of the pre-verification layer: x = hidden + PosEmb[e]; operand and ssq as above
__global__ void mb_input_w16_kernel(const float* __restrict__ src, int lds, const float* __restrict__ posemb, SeqRows sr, MbRows mr,
                                    int d, float* __restrict__ x, int ldx, const float* __restrict__ g, _Float16* __restrict__ xp,
                                    int MT_total, u64* __restrict__ ssq, int n_slots, int slot_stride) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  const int si = find_seq(sr, r);
  const int rr = r - sr.row_off[si];
  const float* h = src + (size_t)(mr.src_row0[si] + rr) * lds;
  const float* e = posemb + (size_t)(mr.e0[si] < 0 ? 0 : mr.e0[si] + rr) * d;
  float4 a0 = {0.f, 0.f, 0.f, 0.f}, b0 = a0;
  if ((int)threadIdx.x * 4 < d) { a0 = *reinterpret_cast<const float4*>(h + threadIdx.x * 4); b0 = *reinterpret_cast<const float4*>(e + threadIdx.x * 4); }
  float ss = 0.f;
  for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
    const bool first = k == (int)threadIdx.x * 4;
    const float4 a = first ? a0 : *reinterpret_cast<const float4*>(h + k), b = first ? b0 : *reinterpret_cast<const float4*>(e + k);
    const float v0 = a.x + b.x, v1 = a.y + b.y, v2 = a.z + b.z, v3 = a.w + b.w;
    *reinterpret_cast<float4*>(x + (size_t)r * ldx + k) = make_float4(v0, v1, v2, v3);
    store_packed4(xp, MT_total, r, k, v0 * g[k], v1 * g[k + 1], v2 * g[k + 2], v3 * g[k + 3]);
    ss += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3;
  }
  ss = block_sum(ss, red);
  ssq_init_row(ssq, n_slots, slot_stride, r, ss);
}

// hidden = x * g * row_scale for R rows (prompt ingestion: feeds M_B's prefix rows)
__global__ void hidden_rows_kernel(const float* __restrict__ x, int ldx, const float* __restrict__ g, const u64* __restrict__ ssq,
                                   int ssq_stride, float inv_dim, float eps, int d, float* __restrict__ out, int ldo) {
  const int r = blockIdx.x;
  const float rs = row_scale(ssq, ssq_stride, r, inv_dim, eps);
  for (int k = threadIdx.x; k < d; k += blockDim.x) out[(size_t)r * ldo + k] = x[(size_t)r * ldx + k] * g[k] * rs;
}

// ------------------------------------------------------------------ weight-streaming small-M GEMM, fused epilogues
// element offsets inside one (sequence, layer) K or V block of the f16 cache (layout in the file header)
__device__ __forceinline__ size_t kcache_index(int h, int hd, int max_seq, int pos, int f) {
  return (((size_t)h * (max_seq >> 4) + (pos >> 4)) * (hd >> 5) + (f >> 5)) * 512 + ((((f & 31) >> 3) << 4) + (pos & 15)) * 8 + (f & 7);
}
__device__ __forceinline__ size_t vcache_index(int h, int hd, int max_seq, int pos, int f) {
  const int p = pos & 31;
  return (((size_t)h * (max_seq >> 5) + (pos >> 5)) * (hd >> 4) + (f >> 4)) * 512 + ((((p & 15) >> 2) << 4) + (f & 15)) * 8 + (p & 3) + ((p >> 4) << 2);
}

struct GemmArgs {
  const u32x4* W;        // packed weights
  const u32x4* X;        // packed f16 operand [kt][mt_total][lane]
  int KT, R, mt0, mt_total, nt_begin;
  int nt_end;            // one past the last output tile (streaming kernel: blocks may overhang it)
  const u64* ssq_in;     // row sums of squares of the operand's source rows (null: no row scale)
  int ssq_stride;
  float inv_dim, eps;
  float* out;            // STORE: [rows][ldo] ; RESID: the residual stream x (read, add, write)
  int ldo, rowmap, G1;
  _Float16* xp_out;      // RESID: next operand f16(x*g_next) ; SWIGLU: f16(act)
  int mt_total_out;
  const float* g_next;
  u64* ssq_out;
  _Float16* qp;          // QKV: attention operand [slot][head][kt][2][lane][8]
  _Float16* kv;          // QKV: cache base of the model
  const float* rope;     // QKV: the model's table [max_seq][hd/2][2] cos, sin by absolute position
  int d, hd, layer, n_layers, max_seq, H;
  // STORE of draft logits: per (row, output tile) candidate of the token choice
  float* pick_val;       // [rows][pick_tiles] best logit (+ Gumbel noise when sampling); null: off
  int* pick_idx;
  int pick_tiles, pick_mode;
  uint64_t pick_seed;
  uint32_t pick_step;
  SeqRows sr;
  // K split across blocks (streaming kernel, KSB > 1): per-block partial sums [group][KSB][NT*MT][64] f32x4
  // and one arrival counter per group of output tiles (zero between launches)
  float* sk_part;
  unsigned* sk_cnt;
};

// Epilogue of one accumulator lane, shared by the GEMM kernels.  Lane l of a 16x16 result tile holds
// tile rows (outputs) 4*(l/16)..+3 of activation row m; s2 holds the same for the partner outputs i+8
// (paired weight layouts: rotation pairs of QKV, gate/up of SwiGLU; lanes with l/16 < 2).  All 64 lanes
// of the tile call this together (the row reductions use wave shuffles).
// ssq_pre: the row's sum of squares (the integer parts added up) if the caller fetched it ahead of time
template <int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& ga, int nt, int m, int l, f32x4 s, f32x4 s2, const u64* ssq_pre = nullptr) {
  const int g4 = l >> 4;
  const bool live = m < ga.R;
  float rs = 1.f;
  if (ga.ssq_in && live)
    rs = ssq_pre ? 1.0f / sqrtf((float)*ssq_pre * SSQ_INV_SCALE * ga.inv_dim + ga.eps) : row_scale(ga.ssq_in, ga.ssq_stride, m, ga.inv_dim, ga.eps);

  if (EPI == EPI_STORE) {
    const int n = nt * 16 + g4 * 4;
    const f32x4 lg = s * rs;
    if (live) {
      float* o = ga.out + (size_t)map_row(ga.sr, ga.rowmap, ga.G1, m) * ga.ldo + n;
      *reinterpret_cast<f32x4*>(o) = lg;
    }
    if (ga.pick_val) {
      // token choice, first stage: best of this tile's 16 vocabulary entries for row m
      // (argmax of the logits, or of logits + Gumbel noise; lowest id wins ties)
      float best = -INFINITY;
      int bi = 0x7fffffff;
      if (live) {
        float g4n[4] = {0.f, 0.f, 0.f, 0.f};
        if (ga.pick_mode) {
          const int si = find_seq(ga.sr, m);
          const int jrow = ga.sr.pos0[si] + (m - ga.sr.row_off[si]) - (ga.sr.len[si] - 1);
          const uint4 bits = vocab_bits(ga.pick_seed, ga.sr.seq[si], ga.pick_step, (uint32_t)(jrow + 1), PURPOSE_DRAFT, (uint32_t)(n >> 2));
          g4n[0] = gumbel(u01(bits.x)); g4n[1] = gumbel(u01(bits.y)); g4n[2] = gumbel(u01(bits.z)); g4n[3] = gumbel(u01(bits.w));
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float v = lg[r] + g4n[r];
          if (v > best) { best = v; bi = n + r; }
        }
      }
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float ov = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
      if (live && g4 == 0) {
        ga.pick_val[(size_t)m * ga.pick_tiles + nt] = best;
        ga.pick_idx[(size_t)m * ga.pick_tiles + nt] = bi;
      }
    }
  } else if (EPI == EPI_RESID) {
    float sq = 0.f;
    if (live) {
      const int n = nt * 16 + g4 * 4;
      float* o = ga.out + (size_t)m * ga.ldo + n;
      const f32x4 xn = *reinterpret_cast<const f32x4*>(o) + s;
      *reinterpret_cast<f32x4*>(o) = xn;
      const float4 gn = *reinterpret_cast<const float4*>(ga.g_next + n);
      store_packed4(ga.xp_out, ga.mt_total_out, m, n, xn[0] * gn.x, xn[1] * gn.y, xn[2] * gn.z, xn[3] * gn.w);
      sq = xn[0] * xn[0] + xn[1] * xn[1] + xn[2] * xn[2] + xn[3] * xn[3];
    }
    sq += __shfl_xor(sq, 16, 64);
    sq += __shfl_xor(sq, 32, 64);
    if (live && g4 == 0) atomicAdd(ga.ssq_out + (size_t)(blockIdx.x % SSQ_SUB) * ga.ssq_stride + m, (u64)(sq * SSQ_SCALE + 0.5f));
  } else if (EPI == EPI_SWIGLU) {
    if (live && g4 < 2) {
      const int f = nt * 8 + g4 * 4;
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float gt = s[r] * rs, up = s2[r] * rs;
        v[r] = gt / (1.0f + expf(-gt)) * up;
      }
      store_packed4(ga.xp_out, ga.mt_total_out, m, f, v[0], v[1], v[2], v[3]);
    }
  } else {  // EPI_QKV
    if (live) {
      const int d = ga.d, hd = ga.hd, half = hd >> 1;
      const int si = find_seq(ga.sr, m);
      const int rl = m - ga.sr.row_off[si];
      const int pos = ga.sr.pos0[si] + rl;
      _Float16* Kc = ga.kv + (((size_t)ga.sr.seq[si] * ga.n_layers + ga.layer) * 2) * (size_t)ga.max_seq * d;
      _Float16* Vt = Kc + (size_t)ga.max_seq * d;
      const int tiles_d = d >> 4;
      typedef _Float16 half4 __attribute__((ext_vector_type(4)));
      if (nt < 2 * tiles_d) {
        if (g4 < 2) {
          const int part = nt / tiles_d;
          const int tq = nt - part * tiles_d;
          const int tph = hd >> 4;
          const int h = tq / tph, tt = tq % tph;
          const int j0 = 8 * tt + 4 * g4;                   // rotation pairs j0..j0+3
          const float* tb = ga.rope + ((size_t)pos * half + j0) * 2;
          float va[4], vb[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float cs = tb[2 * r], sn = tb[2 * r + 1];
            const float x0 = s[r] * rs, x1 = s2[r] * rs;
            va[r] = x0 * cs - x1 * sn;
            vb[r] = x1 * cs + x0 * sn;
          }
          const half4 ha = {(_Float16)va[0], (_Float16)va[1], (_Float16)va[2], (_Float16)va[3]};
          const half4 hb = {(_Float16)vb[0], (_Float16)vb[1], (_Float16)vb[2], (_Float16)vb[3]};
          if (part == 0) {
            // attention operand: [slot][head][kt][2 row tiles][hi|lo][lane][8], lane = 16*(dim%32/8) + row%16
            const int kts = hd >> 5;
            auto qidx = [&](int dim) {
              return ((((size_t)si * ga.H + h) * kts + (dim >> 5)) * 2 + (rl >> 4)) * 1024 + (((dim & 31) >> 3) * 16 + (rl & 15)) * 8 + (dim & 7);
            };
            const half4 la = {(_Float16)(va[0] - (float)ha[0]), (_Float16)(va[1] - (float)ha[1]), (_Float16)(va[2] - (float)ha[2]), (_Float16)(va[3] - (float)ha[3])};
            const half4 lb = {(_Float16)(vb[0] - (float)hb[0]), (_Float16)(vb[1] - (float)hb[1]), (_Float16)(vb[2] - (float)hb[2]), (_Float16)(vb[3] - (float)hb[3])};
            *reinterpret_cast<half4*>(ga.qp + qidx(j0)) = ha;
            *reinterpret_cast<half4*>(ga.qp + qidx(j0) + 512) = la;
            *reinterpret_cast<half4*>(ga.qp + qidx(j0 + half)) = hb;
            *reinterpret_cast<half4*>(ga.qp + qidx(j0 + half) + 512) = lb;
          } else {
            *reinterpret_cast<half4*>(Kc + kcache_index(h, hd, ga.max_seq, pos, j0)) = ha;
            *reinterpret_cast<half4*>(Kc + kcache_index(h, hd, ga.max_seq, pos, j0 + half)) = hb;
          }
        }
      } else {
        const int c0 = (nt - 2 * tiles_d) * 16 + g4 * 4;       // V feature index
        const int h = c0 / hd, f0 = c0 - h * hd;
#pragma unroll
        for (int r = 0; r < 4; ++r) Vt[vcache_index(h, hd, ga.max_seq, pos, f0 + r)] = (_Float16)(s[r] * rs);
      }
    }
  }
}

// X17 = 1 (with MT = 2): the launch covers exactly 17 rows (a full draft window plus the committed
// token).  Only row 16 of the second row tile exists, so its hi and lo parts share ONE extra MFMA: operand
// column 0 = hi of row 16, column 1 = lo of row 16, the other columns zero in registers, and the epilogue
// adds accumulator columns 0 and 1.  That is three MFMAs and 17 fetched operand rows per K step instead
// of four and 32.
// 8-wave blocks are held to 128 VGPRs (4 waves per SIMD) so that two blocks fit a CU.
// HL = operand parts multiplied: 2 = hi and lo tiles (the target model's QKV, gate/up and down GEMMs),
// 1 = hi only (draft and pre-verification layer: two layers deep, their logits stay at 4e-3 of the RMS).
// KSB > 1: K is also split across KSB blocks (block id = group * KSB + slice; a group is NT output tiles).
// Every block of the launch needs the operand rows of its K range, so a matrix with about as many tiles as
// there are CUs (O and down projections) fetches the operand once per tile; with KSB slices of NT = KSB
// tiles each the block count stays and each block fetches 1/KSB of it.  The slices' sums meet in memory
// without a device-scope fence (which writes back and invalidates a whole L2 and costs far more than it
// saves here): each block writes its partial tiles with agent-scope relaxed atomic stores (write-through
// to memory: `sc1`), waits until they have completed (vmcnt 0), and then bumps the group's counter with
// an agent-scope atomic add; the block that sees the other KSB-1 arrivals reads all partials back with
// agent-scope atomic loads (which do not hit in its XCD's L2), adds them in slice order (so the result
// does not depend on which block came last), resets the counter and runs the epilogue.  Nobody waits
// for anybody: a block that is not the last one simply ends.
template <int EPI, int MT, int NT, int WAVES, int U, int TAG, int X17 = 0, int HL = 1, int KSB = 1>
__global__ __launch_bounds__(WAVES * 64, (WAVES == 8 ? (NT >= 5 ? 2 : 4) : 1)) void gemm_w16_kernel(const GemmArgs ga) {
  static_assert(!X17 || MT == 2, "the 17-row form uses two row tiles");
  // partial sums of the waves; more than 64 KB of them are handed over in two halves
  constexpr int RW = (WAVES * NT * MT > 64) ? WAVES / 2 : WAVES;
  static_assert(RW * NT * MT <= 64, "the reduction buffer must fit the 64 KB of static LDS");
  static_assert(KSB <= RW, "the partial sums of the K slices are gathered in the reduction buffer");
  constexpr int NRED = KSB > 1 ? KSB : RW;            // summands per accumulator lane in the epilogue
  __shared__ f32x4 red[RW][NT * MT][64];
  __shared__ unsigned sk_arrived;
  const int grp = blockIdx.x / KSB, ks = blockIdx.x % KSB;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave id as a scalar
  const int nt0 = ga.nt_begin + grp * NT;
  const int KT = ga.KT;
  const int kbeg = (int)((long)ks * KT / KSB), kend = (int)((long)(ks + 1) * KT / KSB);   // this block's K steps
  // K steps are dealt to the block's waves round-robin (wave w takes w, w+WAVES, ...): at any moment
  // the waves of a block, and the blocks sharing a CU, read neighbouring operand tiles, which keeps the
  // operand in the CU's L1 instead of fetching it once per wave from L2
  // steps of this wave: index i -> kt = kbeg + i*WAVES + wave
  const int kb = 0;
  const int ke = (kend - kbeg - wave + WAVES - 1) / WAVES;
  f32x4 acc[NT][MT];
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int b = 0; b < MT; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4* wp[NT];
#pragma unroll
  for (int a = 0; a < NT; ++a) wp[a] = ga.W + (size_t)min(nt0 + a, ga.nt_end - 1) * KT * 64 + lane;   // a tile past the end repeats the last one, unused
  // Operand pointers, one per row tile.  Lanes whose row does not exist read the tile's last live row instead
  // (the same cache lines the live lanes fetch, and their accumulator columns are discarded): the operand
  // traffic scales with the number of rows, not with whole 16-row tiles, and no load is conditional.
  const u32x4* xpb[MT];
#pragma unroll
  for (int b = 0; b < MT; ++b) {
    const int live = min(16, max(1, ga.R - (ga.mt0 + b) * 16));
    xpb[b] = ga.X + (size_t)(ga.mt0 + b) * 128 + min(lane & 15, live - 1) * 4 + (lane >> 4);
  }
  // row 0 of row tile mt0+1: its hi part for even operand columns, its lo part for odd ones
  const u32x4* xp17 = ga.X + (size_t)(ga.mt0 + 1) * 128 + (lane >> 4) + (HL == 2 ? (lane & 1) * 64 : 0);
  const bool x17_live = (lane & 15) < HL;
  const int mtt = ga.mt_total;

  constexpr int BW = X17 ? HL + 1 : MT * HL;           // operand tiles per K step: [row tile][part]
  u32x4 A0[U][NT], A1[U][NT], B0[U][BW], B1[U][BW];
  const u32x4 zero = {0u, 0u, 0u, 0u};
  // The K loop has no branches: a branch around a load makes the compiler wait for every outstanding load
  // where the paths join (the load counter completes in order, and the number of newer loads then differs
  // by path), which would serialise each wave on memory latency.  K steps past the wave's last one re-read
  // its last tile (an L1 hit) and their weights are replaced by zeros before use.
  auto load = [&](u32x4(&A)[U][NT], u32x4(&B)[U][BW], int k0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t kt = (size_t)min(kbeg + (k0 + u) * WAVES + wave, kend - 1);
#pragma unroll
      for (int a = 0; a < NT; ++a) A[u][a] = __builtin_nontemporal_load(wp[a] + kt * 64);
      if (X17) {
#pragma unroll
        for (int h = 0; h < HL; ++h) B[u][h] = xpb[0][(kt * mtt * 2 + h) * 64];
        B[u][HL] = xp17[kt * mtt * 2 * 64];
      } else {
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
          for (int h = 0; h < HL; ++h) B[u][b * HL + h] = xpb[b][(kt * mtt * 2 + h) * 64];
      }
    }
  };
  auto compute = [&](u32x4(&A)[U][NT], u32x4(&B)[U][BW], int k0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool valid = k0 + u < ke;                  // wave-uniform
      half8 bh[BW];
#pragma unroll
      for (int b = 0; b < BW; ++b) bh[b] = __builtin_bit_cast(half8, (X17 && b == HL && !x17_live) ? zero : B[u][b]);
#pragma unroll
      for (int a = 0; a < NT; ++a) {
        const half8 ah = __builtin_bit_cast(half8, valid ? A[u][a] : zero);
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
          for (int h = 0; h < HL; ++h) {
            if (X17 && b == 1 && h > 0) continue;
            acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh[(X17 && b == 1) ? HL : b * HL + h], acc[a][b], 0, 0, 0);
          }
      }
    }
  };
  // Two register sets; each is refilled right after its products were issued, in the same order on every
  // path into the loop, and the scheduler may not move loads across the phase boundaries: the wait before
  // a phase's products then leaves the other set's loads in flight.
  // The epilogue's row scale needs the operand rows' sums of squares: they are requested here, ahead of the
  // weight stream, so that the epilogue does not end the kernel on one more memory round trip.
  constexpr int EIT = (NT * MT * 64 + WAVES * 64 - 1) / (WAVES * 64);     // epilogue items per thread
  u64 ssq_pre[EIT][SSQ_SUB];
#pragma unroll
  for (int it = 0; it < EIT; ++it) {
    const int t = threadIdx.x + it * WAVES * 64;
    const int m = (ga.mt0 + (t >> 6) % MT) * 16 + (t & 15);
    const bool want = ga.ssq_in && t < NT * MT * 64 && m < ga.R;
#pragma unroll
    for (int i = 0; i < SSQ_SUB; ++i) ssq_pre[it][i] = want ? ga.ssq_in[(size_t)i * ga.ssq_stride + m] : 0ull;
  }
  __builtin_amdgcn_sched_barrier(0);
  load(A0, B0, kb);
  __builtin_amdgcn_sched_barrier(0);
  for (int k0 = kb; k0 < ke; k0 += 2 * U) {
    load(A1, B1, k0 + U);
    __builtin_amdgcn_sched_barrier(0);
    compute(A0, B0, k0);
    __builtin_amdgcn_sched_barrier(0);
    load(A0, B0, k0 + 2 * U);
    __builtin_amdgcn_sched_barrier(0);
    compute(A1, B1, k0 + U);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (RW < WAVES) {
    if (wave >= RW) {
#pragma unroll
      for (int a = 0; a < NT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) red[wave - RW][a * MT + b][lane] = acc[a][b];
    }
    __syncthreads();
    if (wave < RW) {
#pragma unroll
      for (int a = 0; a < NT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) acc[a][b] += red[wave][a * MT + b][lane];
    }
    __syncthreads();
  }
  if (wave < RW) {
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
      for (int b = 0; b < MT; ++b) red[wave][a * MT + b][lane] = acc[a][b];
  }
  __syncthreads();
  if (KSB > 1) {
    u64* part = reinterpret_cast<u64*>(ga.sk_part);
#pragma unroll
    for (int it = 0; it < EIT; ++it) {
      const int t = threadIdx.x + it * WAVES * 64;
      if (t < NT * MT * 64) {
        f32x4 p = red[0][t >> 6][t & 63];
#pragma unroll
        for (int w = 1; w < RW; ++w) p += red[w][t >> 6][t & 63];
        u64* dst = part + ((size_t)(grp * KSB + ks) * NT * MT * 64 + t) * 2;
        const float2 lo = {p[0], p[1]}, hi = {p[2], p[3]};
        __hip_atomic_store(dst, __builtin_bit_cast(u64, lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(dst + 1, __builtin_bit_cast(u64, hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    PACER_WAIT_VMCNT0();   // this wave's write-through stores have completed
    __syncthreads();
    if (threadIdx.x == 0) sk_arrived = __hip_atomic_fetch_add(ga.sk_cnt + grp, 1u, PACER_HO_ORDER, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sk_arrived != KSB - 1) return;
    if (threadIdx.x == 0) __hip_atomic_store(ga.sk_cnt + grp, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int it = 0; it < EIT; ++it) {
      const int t = threadIdx.x + it * WAVES * 64;
      if (t < NT * MT * 64) {
#pragma unroll
        for (int k = 0; k < KSB; ++k) {
          const u64* src = part + ((size_t)(grp * KSB + k) * NT * MT * 64 + t) * 2;
          const float2 lo = __builtin_bit_cast(float2, __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          const float2 hi = __builtin_bit_cast(float2, __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          red[k][t >> 6][t & 63] = f32x4{lo.x, lo.y, hi.x, hi.y};
        }
      }
    }
    __syncthreads();
  }

  // Epilogue.  One wave-sized group of threads per (tile a, row tile b); thread l of the group owns the
  // accumulator lane l: activation row m = 16*(mt0+b) + l%16, tile rows 4*(l/16)..+3.
#pragma unroll
  for (int it = 0; it < EIT; ++it) {
    const int t = threadIdx.x + it * WAVES * 64;
    if (t >= NT * MT * 64) break;
    u64 ssq_sum = 0;
#pragma unroll
    for (int i = 0; i < SSQ_SUB; ++i) ssq_sum += ssq_pre[it][i];
    const int l = t & 63, ab = t >> 6;
    const int a = ab / MT, b = ab % MT;
    const int g4 = l >> 4;
    const int m = (ga.mt0 + b) * 16 + (l & 15);
    const int nt = nt0 + a;
    if (nt >= ga.nt_end) continue;
    const bool paired = (EPI == EPI_SWIGLU) || (EPI == EPI_QKV);
    f32x4 s = red[0][ab][l];
#pragma unroll
    for (int w = 1; w < NRED; ++w) s += red[w][ab][l];
    f32x4 s2 = {0.f, 0.f, 0.f, 0.f};                   // partner rows i+8 (paired layouts, threads with g4 < 2)
    if (paired && g4 < 2) {
      s2 = red[0][ab][l + 32];
#pragma unroll
      for (int w = 1; w < NRED; ++w) s2 += red[w][ab][l + 32];
    }
    if (X17 && HL == 2 && b == 1 && (l & 15) == 0) {   // row 16: hi product in column 0, lo product in column 1
#pragma unroll
      for (int w = 0; w < NRED; ++w) s += red[w][ab][l + 1];
      if (paired && g4 < 2) {
#pragma unroll
        for (int w = 0; w < NRED; ++w) s2 += red[w][ab][l + 33];
      }
    }
    gemm_epilogue<EPI>(ga, nt, m, l, s, s2, &ssq_sum);
  }
}

// ------------------------------------------------------------------ wide GEMM: more than 32 rows
// Batched verification puts up to 16 x 17 rows through the target model; at that width the product is
// bound by the matrix units and by operand delivery, not by the weight stream, so the roles change:
//   block  = KS K-slices x 4 waves; a slice's 4 waves own 4*NTW output tiles x MTB row tiles over
//            their 1/KS of K, walked in super-steps of KC = 4/KS K steps; the slices' sums meet in LDS
//   weights: each wave streams its own NTW tiles into registers, 4 K steps ahead
//   operand: a slice's MTB*HL tiles of a super-step are fetched once (two super-steps ahead), written
//            to LDS in MFMA lane order (double buffered, one barrier per super-step) and read by the
//            slice's four waves, so each operand byte feeds 4*NTW tiles and each weight byte MTB*HL MFMAs
// KS > 1 is for matrices with few output tiles (O and down projections): it is what puts 8 waves on a CU
// when there are fewer blocks than CUs, and a wave alone on its SIMD cannot hide the weight stream's latency.
// Blocks that share weights (same output tiles, different rows) get consecutive slots on one XCD
// (block id mod 8 picks the XCD), so the weight stream of the later ones comes from that XCD's L2
// (measured: 1.2 to 1.5 x the weight bytes from HBM with three row groups).
// The K loop has no branches and no conditional loads (a branch makes the compiler wait for every
// outstanding load at the join, which serialises the pipeline on memory latency): tiles or K steps that
// do not exist are replaced by the nearest one that does, and their products are never stored.
// Requires KT % (4*KS) == 0.
template <int EPI, int NTW, int MTB, int HL, int TAG, int KS>
__global__ __launch_bounds__(256 * KS, (KS == 1 ? 2 : 1)) void gemm_wide_kernel(const GemmArgs ga, int n_tiles, int n_groups, int row_groups) {
  constexpr int UA = 4, KC = UA / KS, BT = MTB * HL, BI = (BT + 3) / 4;
  __shared__ u32x4 Bs[KS][2][KC][BI * 4][64];
  static_assert(KS == 1 || 4 * NTW * MTB <= KS * 2 * KC * BI * 4, "slice sums reuse the operand buffers");
  // wave-uniform ids as scalars, so that tile pointers and K offsets live in scalar registers
  const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wave = wid & 3, ks = wid >> 2, lane = threadIdx.x & 63;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int rg = slot % row_groups, ng = (slot / row_groups) * 8 + xcd;
  if (ng >= n_groups) return;
  const int mtt = ga.mt_total;
  const int mt_lo = mtt * rg / row_groups;
  const int mtb = mtt * (rg + 1) / row_groups - mt_lo;       // row tiles of this block, 1..MTB
  const int nt0 = ga.nt_begin + (ng * 4 + wave) * NTW;
  const int nt_end = ga.nt_begin + n_tiles;
  const int KT = ga.KT, kb = ks * (KT / KS), ke = kb + KT / KS;

  f32x4 acc[NTW][MTB];
#pragma unroll
  for (int a = 0; a < NTW; ++a)
#pragma unroll
    for (int b = 0; b < MTB; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4* wp[NTW];
#pragma unroll
  for (int a = 0; a < NTW; ++a) wp[a] = ga.W + (size_t)min(nt0 + a, nt_end - 1) * KT * 64 + lane;
  // operand staging: wave w copies tile-parts w, w+4, ...; lane 16g+j reads row j's bytes 16g..16g+15
  const u32x4* xsrc[BI];
#pragma unroll
  for (int it = 0; it < BI; ++it) {
    const int tp = min(it * 4 + wave, BT - 1), b = min(tp / HL, mtb - 1), h = tp % HL;
    xsrc[it] = ga.X + ((size_t)(mt_lo + b) * 2 + h) * 64 + (lane & 15) * 4 + (lane >> 4);
  }
  const size_t xstep = (size_t)mtt * 128;                      // operand elements (16 B) per K step
  u32x4 Areg[UA][NTW], Breg[KC][BI];
  auto loadA = [&](u32x4(&A)[NTW], int k) {                    // plain loads: row groups sharing these tiles find them in L2
    const size_t o = (size_t)min(k, ke - 1) * 64;
#pragma unroll
    for (int a = 0; a < NTW; ++a) A[a] = wp[a][o];
  };
  auto loadB = [&](u32x4(&B)[BI], int k) {
    const size_t o = (size_t)min(k, ke - 1) * xstep;
#pragma unroll
    for (int it = 0; it < BI; ++it) B[it] = xsrc[it][o];
  };
  auto storeB = [&](int buf) {
#pragma unroll
    for (int j = 0; j < KC; ++j)
#pragma unroll
      for (int it = 0; it < BI; ++it) Bs[ks][buf][j][it * 4 + wave][lane] = Breg[j][it];
  };
  // Prologue: operand of super-step 0 into LDS, of super-step 1 into registers; weights of 4 steps.
  // Loads are issued in the order the loop issues them (operand, then weights step by step) and the
  // scheduler is told not to move them (sched_barrier): the load counter completes in order, so a wait
  // for an older load can leave the newer ones in flight only if the order is the same on every path into
  // the loop.  Left to itself the compiler gathered all loads at the end of the loop body and waited for
  // every one of them at the top (1.3 to 1.5 x slower).
#pragma unroll
  for (int j = 0; j < KC; ++j) loadB(Breg[j], kb + j);
  storeB(0);
#pragma unroll
  for (int j = 0; j < KC; ++j) loadB(Breg[j], kb + KC + j);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < UA; ++u) loadA(Areg[u], kb + u);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  int buf = 0;
  for (int k0 = kb; k0 < ke; k0 += UA) {
#pragma unroll
    for (int ss = 0; ss < UA / KC; ++ss) {
      storeB(buf ^ 1);                                         // operand of the next super-step
#pragma unroll
      for (int j = 0; j < KC; ++j) loadB(Breg[j], k0 + ss * KC + 2 * KC + j);
      __builtin_amdgcn_sched_barrier(0);
      // operand tiles of K step j+1 are read from LDS before the products of step j are issued (two register sets)
      u32x4 bfr[2][BT];
#pragma unroll
      for (int t = 0; t < BT; ++t) bfr[0][t] = Bs[ks][buf][0][t][lane];
#pragma unroll
      for (int j = 0; j < KC; ++j) {
        const int u = ss * KC + j;
        if (j + 1 < KC) {
#pragma unroll
          for (int t = 0; t < BT; ++t) bfr[(j + 1) & 1][t] = Bs[ks][buf][j + 1][t][lane];
        }
        __builtin_amdgcn_sched_barrier(0);
        half8 af[NTW];
#pragma unroll
        for (int a = 0; a < NTW; ++a) af[a] = __builtin_bit_cast(half8, Areg[u][a]);
#pragma unroll
        for (int t = 0; t < BT; ++t)
#pragma unroll
          for (int a = 0; a < NTW; ++a)
            acc[a][t / HL] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[a], __builtin_bit_cast(half8, bfr[j & 1][t]), acc[a][t / HL], 0, 0, 0);
        // the step's weight registers are free now: refill them for the step UA ahead (after the products, so
        // that the loads land in the same registers and need no copies at the loop's back edge)
        loadA(Areg[u], k0 + UA + u);
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
      buf ^= 1;
    }
  }
  if (KS > 1) {
    // slices 1.. hand their sums to slice 0 through the (now idle) operand buffers, one slice at a time, in slice order
    f32x4* red = reinterpret_cast<f32x4*>(&Bs[0][0][0][0][0]);
#pragma unroll
    for (int s = 1; s < KS; ++s) {
      if (ks == s) {
#pragma unroll
        for (int a = 0; a < NTW; ++a)
#pragma unroll
          for (int b = 0; b < MTB; ++b) red[((wave * NTW + a) * MTB + b) * 64 + lane] = acc[a][b];
      }
      __syncthreads();
      if (ks == 0) {
#pragma unroll
        for (int a = 0; a < NTW; ++a)
#pragma unroll
          for (int b = 0; b < MTB; ++b) acc[a][b] += red[((wave * NTW + a) * MTB + b) * 64 + lane];
      }
      __syncthreads();
    }
    if (ks > 0) return;
  }

  constexpr bool paired = (EPI == EPI_SWIGLU) || (EPI == EPI_QKV);
#pragma unroll
  for (int a = 0; a < NTW; ++a) {
    if (nt0 + a >= nt_end) continue;
#pragma unroll
    for (int b = 0; b < MTB; ++b) {
      if (b >= mtb) continue;
      const f32x4 s = acc[a][b];
      f32x4 s2 = {0.f, 0.f, 0.f, 0.f};
      if (paired) {
#pragma unroll
        for (int r = 0; r < 4; ++r) s2[r] = __shfl(s[r], (lane + 32) & 63, 64);
      }
      gemm_epilogue<EPI>(ga, nt0 + a, (mt_lo + b) * 16 + (lane & 15), lane, s, s2);
    }
  }
}

// ------------------------------------------------------------------ wide GEMM, few output tiles: K slices across blocks
// The O and down projections of a batched verification pass (about 100..200 rows) have only a few hundred
// output tiles; with the kernel above their blocks either cover few rows (the weights are then read once per
// row group) or are too few for the CUs.  Here a block is 8 waves that share ONE operand stage (wave w owns
// NTW output tiles, all MTB row tiles of the block), so an operand byte feeds 8*NTW tiles, and K is split
// over KSB blocks whose partial tiles are added by the block that finishes last (write-through stores,
// counter, L2-bypassing loads: see gemm_w16_kernel).  Measured at d 5120, K 13824, 128 rows: 53 us against
// 75 us for the best shape of the kernel above; 144 rows: 63 against 80 us.
//   grid = ceil(groups / 8) * 8 * row_groups * KSB, block id -> (XCD = id % 8, then row group, K slice, group)
//   dynamic LDS = 2 * KC * MTB * HL KiB (operand of two super-steps of KC K steps)
// Requires KT % 4 == 0 and KT / 4 >= KSB.
template <int EPI, int NTW, int MTB, int HL, int TAG, int KC, int KSB>
__global__ __launch_bounds__(512, 1) void gemm_wide8_kernel(const GemmArgs ga, int n_tiles, int n_groups, int row_groups) {
  constexpr int WV = 8, UA = 4, BT = MTB * HL, ITS = (KC * BT + WV - 1) / WV;
  static_assert(UA % KC == 0, "super-steps divide the weight prefetch depth");
  extern __shared__ __align__(16) u32x4 wide8_stage[];     // [2][KC][BT][64]
  __shared__ unsigned arrived;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int rg = slot % row_groups, ksl = (slot / row_groups) % KSB, ng = (slot / (row_groups * KSB)) * 8 + xcd;
  if (ng >= n_groups) return;
  const int mtt = ga.mt_total;
  const int mt_lo = mtt * rg / row_groups;
  const int mtb = mtt * (rg + 1) / row_groups - mt_lo;       // row tiles of this block, 1..MTB
  const int nt0 = ga.nt_begin + (ng * WV + wave) * NTW;
  const int nt_end = ga.nt_begin + n_tiles;
  const int units = ga.KT / UA;
  const int kb = (int)((long)ksl * units / KSB) * UA, ke = (int)((long)(ksl + 1) * units / KSB) * UA;

  f32x4 acc[NTW][MTB];
#pragma unroll
  for (int a = 0; a < NTW; ++a)
#pragma unroll
    for (int b = 0; b < MTB; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4* wp[NTW];
#pragma unroll
  for (int a = 0; a < NTW; ++a) wp[a] = ga.W + (size_t)min(nt0 + a, nt_end - 1) * ga.KT * 64 + lane;
  // operand staging: the KC*BT tile-parts of a super-step are dealt to the 8 waves round-robin; a part past
  // the last repeats it (same data to the same LDS slot), a row tile past the block's last repeats that one
  const u32x4* xsrc[ITS];
  int xj[ITS], xdst[ITS];
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int ti = min(it * WV + wave, KC * BT - 1), j = ti / BT, t = ti % BT;
    const int b = min(t / HL, mtb - 1), h = t % HL;
    xsrc[it] = ga.X + ((size_t)(mt_lo + b) * 2 + h) * 64 + (lane & 15) * 4 + (lane >> 4);
    xj[it] = j;
    xdst[it] = (j * BT + t) * 64 + lane;
  }
  const size_t xstep = (size_t)mtt * 128;                    // operand elements (16 B) per K step
  u32x4 Areg[UA][NTW], Breg[ITS];
  auto loadA = [&](u32x4(&A)[NTW], int k) {
    const size_t o = (size_t)min(k, ke - 1) * 64;
#pragma unroll
    for (int a = 0; a < NTW; ++a) A[a] = wp[a][o];
  };
  auto loadB = [&](int k) {
#pragma unroll
    for (int it = 0; it < ITS; ++it) Breg[it] = xsrc[it][(size_t)min(k + xj[it], ke - 1) * xstep];
  };
  auto storeB = [&](int buf) {
#pragma unroll
    for (int it = 0; it < ITS; ++it) wide8_stage[(size_t)buf * KC * BT * 64 + xdst[it]] = Breg[it];
  };
  // same load order in the prologue and in the loop, pinned (see gemm_wide_kernel)
  loadB(kb);
  storeB(0);
  loadB(kb + KC);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < UA; ++u) loadA(Areg[u], kb + u);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  int buf = 0;
  for (int k0 = kb; k0 < ke; k0 += UA) {
#pragma unroll
    for (int ss = 0; ss < UA / KC; ++ss) {
      storeB(buf ^ 1);                                       // operand of the next super-step
      loadB(k0 + ss * KC + 2 * KC);
      __builtin_amdgcn_sched_barrier(0);
      // The operand tiles of K step j+1 are read from LDS into a second register set before the products of
      // step j are issued (with one set the compiler reads a tile, waits, multiplies, reads the next into the
      // same registers: the LDS latency then shows once per tile and the matrix unit idles two thirds of the time).
      u32x4 bfr[2][BT];
      {
        const u32x4* bsrc = wide8_stage + ((size_t)(buf * KC) * BT) * 64 + lane;
#pragma unroll
        for (int t = 0; t < BT; ++t) bfr[0][t] = bsrc[t * 64];
      }
#pragma unroll
      for (int j = 0; j < KC; ++j) {
        const int u = ss * KC + j;
        if (j + 1 < KC) {
          const u32x4* bsrc = wide8_stage + ((size_t)(buf * KC + j + 1) * BT) * 64 + lane;
#pragma unroll
          for (int t = 0; t < BT; ++t) bfr[(j + 1) & 1][t] = bsrc[t * 64];
        }
        __builtin_amdgcn_sched_barrier(0);
        half8 af[NTW];
#pragma unroll
        for (int a = 0; a < NTW; ++a) af[a] = __builtin_bit_cast(half8, Areg[u][a]);
#pragma unroll
        for (int t = 0; t < BT; ++t) {
          const half8 bf = __builtin_bit_cast(half8, bfr[j & 1][t]);
#pragma unroll
          for (int a = 0; a < NTW; ++a) acc[a][t / HL] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[a], bf, acc[a][t / HL], 0, 0, 0);
        }
        loadA(Areg[u], k0 + UA + u);                         // refill after the products: same registers, no copies
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
      buf ^= 1;
    }
  }
  if (KSB > 1) {
    // partial tiles of this K slice, written through to memory; whoever arrives last adds all slices in slice order
    u64* part = reinterpret_cast<u64*>(ga.sk_part);
    const size_t per_block = (size_t)WV * NTW * MTB * 64 * 2;          // 8-byte words per block
    const size_t gidx = (size_t)ng * row_groups + rg;
    u64* mine = part + (gidx * KSB + ksl) * per_block + ((size_t)wave * NTW * MTB * 64 + lane) * 2;
#pragma unroll
    for (int a = 0; a < NTW; ++a)
#pragma unroll
      for (int b = 0; b < MTB; ++b) {
        const float2 lo = {acc[a][b][0], acc[a][b][1]}, hi = {acc[a][b][2], acc[a][b][3]};
        u64* d = mine + (size_t)(a * MTB + b) * 128;
        __hip_atomic_store(d, __builtin_bit_cast(u64, lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(d + 1, __builtin_bit_cast(u64, hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    PACER_WAIT_VMCNT0();   // this wave's write-through stores have completed
    __syncthreads();
    if (threadIdx.x == 0) arrived = __hip_atomic_fetch_add(ga.sk_cnt + gidx, 1u, PACER_HO_ORDER, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (arrived != KSB - 1) return;
    if (threadIdx.x == 0) __hip_atomic_store(ga.sk_cnt + gidx, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int a = 0; a < NTW; ++a)
#pragma unroll
      for (int b = 0; b < MTB; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KSB; ++s) {
      const u64* src = part + (gidx * KSB + s) * per_block + ((size_t)wave * NTW * MTB * 64 + lane) * 2;
      u64 v0[NTW][MTB], v1[NTW][MTB];
#pragma unroll
      for (int a = 0; a < NTW; ++a)
#pragma unroll
        for (int b = 0; b < MTB; ++b) {
          v0[a][b] = __hip_atomic_load(src + (size_t)(a * MTB + b) * 128, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          v1[a][b] = __hip_atomic_load(src + (size_t)(a * MTB + b) * 128 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
      for (int a = 0; a < NTW; ++a)
#pragma unroll
        for (int b = 0; b < MTB; ++b) {
          const float2 lo = __builtin_bit_cast(float2, v0[a][b]), hi = __builtin_bit_cast(float2, v1[a][b]);
          acc[a][b] += f32x4{lo.x, lo.y, hi.x, hi.y};
        }
    }
  }
  constexpr bool paired = (EPI == EPI_SWIGLU) || (EPI == EPI_QKV);
#pragma unroll
  for (int a = 0; a < NTW; ++a) {
    if (nt0 + a >= nt_end) continue;
#pragma unroll
    for (int b = 0; b < MTB; ++b) {
      if (b >= mtb) continue;
      const f32x4 s = acc[a][b];
      f32x4 s2 = {0.f, 0.f, 0.f, 0.f};
      if (paired) {
#pragma unroll
        for (int r = 0; r < 4; ++r) s2[r] = __shfl(s[r], (lane + 32) & 63, 64);
      }
      gemm_epilogue<EPI>(ga, nt0 + a, (mt_lo + b) * 16 + (lane & 15), lane, s, s2);
    }
  }
}

// ------------------------------------------------------------------ MFMA attention over the f16 KV cache
// grid (key splits, heads, sequences), 8 waves per block.  A block owns `kps` keys of one head; its
// waves take the 32-key groups of that range round-robin, each running an online softmax in registers:
//   scores  S^T[key][row] = K[key][:] . Q[row][:]   (A = K tile straight from the cache, B = Q operand)
//   values  O^T[dim][row] += V^T[dim][keys] P^T[keys][row]; the probabilities leave the first MFMA in
//           exactly the lane layout the second one wants for B (contraction index = the 8 keys a lane
//           holds), and V^T rows are contiguous along keys.
// The 8 wave states meet in LDS (dynamic, 8 x live rows x (HD + 4) floats) and are combined in one pass.
// With one split the block writes the f16 operand of the O projection directly; with several, each block
// writes a partial (un-normalised values, running max, running sum per row) and the block of a (head,
// sequence, row tile) that arrives last combines them, in split order.  The hand-over needs no device-scope
// fence (see gemm_w16_kernel): write-through stores, a wait for their completion, an agent-scope counter,
// and loads that bypass the reader's L2.  `cnt` holds one counter per (sequence slot, head, row-tile half),
// zero between launches.
// QL = 2: the query operand is used as hi + lo (target model), 1: hi only.
template <int HD, int MT, int QL>
__global__ __launch_bounds__(512) void attn_mfma_kernel(const _Float16* __restrict__ qp, const _Float16* __restrict__ kv, int layer,
                                                        int n_layers, int max_seq, int d, SeqRows sr, int kps, int S, int H,
                                                        float* __restrict__ part, _Float16* __restrict__ xp_out, int MT_total_out,
                                                        int rt_split, unsigned* __restrict__ cnt) {
  constexpr int KTS = HD / 32, DTS = HD / 16, NW = 8;
  __shared__ unsigned arrived;
  extern __shared__ __align__(16) float att_state[];   // [8 waves][live rows][HD + 4]: values, running max, running sum
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4, j = lane & 15;
  // rt_split (MT == 1 launches only): two blocks per key range, one per 16-row tile of the sequence
  const int rt = rt_split ? (int)(blockIdx.x & 1) : 0;
  const int split = rt_split ? (int)(blockIdx.x >> 1) : (int)blockIdx.x, h = blockIdx.y, si = blockIdx.z;
  const int r0 = sr.row_off[si] + rt * 16, pos0 = sr.pos0[si];
  const int n_keys = pos0 + sr.row_off[si + 1] - sr.row_off[si];
  const int Rs = sr.row_off[si + 1] - r0;                // rows from this block's first one to the sequence's last
  const int n_split = (n_keys + kps - 1) / kps;
  if (split >= n_split || Rs <= 0) return;
  const int ks_begin = split * kps, ks_end = min(n_keys, ks_begin + kps);
  const _Float16* Kc = kv + (((size_t)sr.seq[si] * n_layers + layer) * 2) * (size_t)max_seq * d + (size_t)h * HD * max_seq;
  const _Float16* Vt = Kc + (size_t)max_seq * d;
  const float scale = 1.0f / sqrtf((float)HD);
  typedef _Float16 half4 __attribute__((ext_vector_type(4)));

  half8 q[KTS][MT][QL];
#pragma unroll
  for (int kt = 0; kt < KTS; ++kt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int pq = 0; pq < QL; ++pq)
        q[kt][mt][pq] = *reinterpret_cast<const half8*>(qp + (((((size_t)si * H + h) * KTS + kt) * 2 + rt + mt) * 2 + pq) * 512 + lane * 8);
  f32x4 acc[DTS][MT];
  float mrun[MT], lrun[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    mrun[mt] = -INFINITY;
    lrun[mt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DTS; ++dt) acc[dt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // One 32-key group = two 16-key K tiles x KTS feature groups, and DTS fragments of V^T.  K and V each have
  // one register set; a set is refilled for the wave's next group as soon as its last product was issued
  // (K after the scores, V after the values), so each load has half a step of this wave's arithmetic, and
  // the other waves, to hide behind.  The loop has no branches and the loads keep their program order
  // (sched_barrier): a wait for K then leaves the V loads in flight and vice versa.  The step after the
  // wave's last one re-reads the last group (cache hits, unused).
  // Cache slots of positions not written yet hold zeros or old finite values (the cache is cleared when it is
  // bound), so their zero probabilities contribute nothing.
  auto load_k = [&](int kk, half8(&ka)[2][KTS]) {
    const _Float16* kt0 = Kc + (size_t)(kk >> 4) * (KTS * 512) + lane * 8;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kt = 0; kt < KTS; ++kt) ka[t][kt] = *reinterpret_cast<const half8*>(kt0 + (t * KTS + kt) * 512);
  };
  auto load_v = [&](int kk, half8(&va)[DTS]) {
    const _Float16* vg = Vt + (size_t)(kk >> 5) * (DTS * 512) + lane * 8;
#pragma unroll
    for (int dt = 0; dt < DTS; ++dt) va[dt] = *reinterpret_cast<const half8*>(vg + dt * 512);
  };
  // scores of one group for row tile mt -> probabilities (f16, in the lane layout the value product wants
  // for B) and the rescale factor of the running state
  auto scores = [&](int kk, int mt, half8(&ka)[2][KTS], half8& pb, float& corr) {
    f32x4 st[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt = 0; kt < KTS; ++kt)
#pragma unroll
        for (int pq = 0; pq < QL; ++pq) sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][kt], q[kt][mt][pq], sacc, 0, 0, 0);
      st[t] = sacc;
    }
    const int pos = pos0 + (rt + mt) * 16 + j;         // this lane's query row
    float sv[8];
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int key = kk + 16 * t + 4 * g + r;
        const float v = (key <= pos && key < n_keys) ? st[t][r] * scale : -INFINITY;
        sv[t * 4 + r] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mn = fmaxf(mrun[mt], mx);
    float ps = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float pe = (mn == -INFINITY) ? 0.f : expf(sv[e] - mn);
      ps += pe;
      pb[e] = (_Float16)pe;
    }
    ps += __shfl_xor(ps, 16, 64);
    ps += __shfl_xor(ps, 32, 64);
    corr = (mrun[mt] == -INFINITY) ? 0.f : expf(mrun[mt] - mn);
    lrun[mt] = lrun[mt] * corr + ps;
    mrun[mt] = mn;
  };
  {
    const int wv = __builtin_amdgcn_readfirstlane(wave);           // scalar: the loop below is uniform per wave
    const int first = ks_begin + 32 * wv;
    const int G = first < ks_end ? (ks_end - first + 32 * NW - 1) / (32 * NW) : 0;
    auto values = [&](half8(&va)[DTS], half8(&pb)[MT], float(&corr)[MT]) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int dt = 0; dt < DTS; ++dt) {
          acc[dt][mt] *= corr[mt];
          acc[dt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va[dt], pb[mt], acc[dt][mt], 0, 0, 0);
        }
    };
    auto key_of = [&](int gi) { return first + min(gi, G - 1) * (32 * NW); };
    if (G > 0) {
      half8 ka[2][KTS], va[DTS];
      __builtin_amdgcn_sched_barrier(0);
      load_k(first, ka);
      __builtin_amdgcn_sched_barrier(0);
      load_v(first, va);
      __builtin_amdgcn_sched_barrier(0);
      for (int gi = 0; gi < G; ++gi) {
        const int kk = key_of(gi), kn = key_of(gi + 1);
        half8 pb[MT];
        float corr[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) scores(kk, mt, ka, pb[mt], corr[mt]);
        __builtin_amdgcn_sched_barrier(0);
        load_k(kn, ka);
        __builtin_amdgcn_sched_barrier(0);
        values(va, pb, corr);
        __builtin_amdgcn_sched_barrier(0);
        load_v(kn, va);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // Merge of the 8 wave states: every wave writes its live rows (values, running max, running sum) to LDS
  // once, then each thread combines the 8 states of one (row, 4 dims) group and writes the result.  One
  // barrier (a pairwise tree over the MFMA tiles took six per row tile and 1.4 to 4 us).
  const int rcap = min(Rs, MT * 16);
  float* st = att_state;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int rl = mt * 16 + j;
    if (rl < rcap) {
      float* o = st + (size_t)(wave * rcap + rl) * (HD + 4);
#pragma unroll
      for (int dt = 0; dt < DTS; ++dt) *reinterpret_cast<f32x4*>(o + dt * 16 + 4 * g) = acc[dt][mt];
      if (g == 0) { o[HD] = mrun[mt]; o[HD + 1] = lrun[mt]; }
    }
  }
  __syncthreads();
  for (int o4 = threadIdx.x; o4 < rcap * (HD / 4); o4 += NW * 64) {
    const int rl = o4 / (HD / 4), d4 = (o4 % (HD / 4)) * 4;
    const float* p = st + (size_t)rl * (HD + 4);
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, p[(size_t)w * rcap * (HD + 4) + HD]);
    float L = 0.f;
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float* pw = p + (size_t)w * rcap * (HD + 4);
      const float m = pw[HD];
      const float wt = (m == -INFINITY) ? 0.f : expf(m - M);
      L += pw[HD + 1] * wt;
      a += *reinterpret_cast<const f32x4*>(pw + d4) * wt;
    }
    if (n_split == 1) {
      const float inv = 1.0f / L;
      store_packed4(xp_out, MT_total_out, r0 + rl, h * HD + d4, a[0] * inv, a[1] * inv, a[2] * inv, a[3] * inv);
    } else {
      // several splits: un-normalised partial (values, running max, running sum), written through to memory
      u64* o = reinterpret_cast<u64*>(part + (((size_t)(r0 + rl) * H + h) * S + split) * (HD + 2));
      const float2 a01 = {a[0], a[1]}, a23 = {a[2], a[3]}, ml = {M, L};
      __hip_atomic_store(o + d4 / 2, __builtin_bit_cast(u64, a01), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(o + d4 / 2 + 1, __builtin_bit_cast(u64, a23), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (d4 == 0) __hip_atomic_store(o + HD / 2, __builtin_bit_cast(u64, ml), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (n_split == 1) return;
  PACER_WAIT_VMCNT0();   // this wave's write-through stores have completed
  __syncthreads();
  unsigned* my_cnt = cnt + ((size_t)si * H + h) * 2 + rt;
  if (threadIdx.x == 0) arrived = __hip_atomic_fetch_add(my_cnt, 1u, PACER_HO_ORDER, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (arrived != (unsigned)(n_split - 1)) return;
  if (threadIdx.x == 0) __hip_atomic_store(my_cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  // last block of this (sequence, head, row tile): combine the splits, eight at a time (all loads of a
  // batch are issued before the first is used; a split past the last repeats it and is skipped)
  for (int o4 = threadIdx.x; o4 < rcap * (HD / 4); o4 += NW * 64) {
    const int rl = o4 / (HD / 4), d4 = (o4 % (HD / 4)) * 4;
    const u64* p = reinterpret_cast<const u64*>(part + ((size_t)(r0 + rl) * H + h) * S * (HD + 2));
    float M = -INFINITY, L = 0.f;
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < n_split; c0 += 8) {
      u64 ml[8], v01[8], v23[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const u64* pc = p + (size_t)min(c0 + i, n_split - 1) * (HD / 2 + 1);
        ml[i] = __hip_atomic_load(pc + HD / 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        v01[i] = __hip_atomic_load(pc + d4 / 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        v23[i] = __hip_atomic_load(pc + d4 / 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      float Mb = M;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (c0 + i < n_split) Mb = fmaxf(Mb, __builtin_bit_cast(float2, ml[i]).x);
      const float keep = (M == -INFINITY) ? 0.f : expf(M - Mb);
      L *= keep;
      a *= keep;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float2 mli = __builtin_bit_cast(float2, ml[i]);
        const float w = (c0 + i < n_split && mli.x != -INFINITY) ? expf(mli.x - Mb) : 0.f;
        const float2 x01 = __builtin_bit_cast(float2, v01[i]), x23 = __builtin_bit_cast(float2, v23[i]);
        L += mli.y * w;
        a[0] += x01.x * w; a[1] += x01.y * w; a[2] += x23.x * w; a[3] += x23.y * w;
      }
      M = Mb;
    }
    const float inv = 1.0f / L;
    store_packed4(xp_out, MT_total_out, r0 + rl, h * HD + d4, a[0] * inv, a[1] * inv, a[2] * inv, a[3] * inv);
  }
}

// ------------------------------------------------------------------ tail of a draft forward
// one block per listed sequence: hidden state h = x * g_final * row_scale into the ring, and the token
// = best of the per-tile candidates the LM-head GEMM left.  With E != null the block goes on to what the next draft
// step would start with, the embedding of the token it has just chosen (row si of next.x, operand, sums of
// squares): a launch less per draft step.  The host skips its embedding launch only if that step really comes next.
__global__ void draft_tail_kernel(const float* x, int ldx, const float* __restrict__ g, const u64* ssq,
                                  int ssq_stride, float inv_dim, float eps, int d, float* __restrict__ hidden, const float* __restrict__ pick_val,
                                  const int* __restrict__ pick_idx, int pick_tiles, int* __restrict__ draft_tok, PickArgs pa, int G1,
                                  const uint16_t* __restrict__ E, EmbedOut next, int V, int* host_bad) {
  __shared__ float redv[16];
  __shared__ int redi[16];
  __shared__ float red[16];
  const int si = blockIdx.x, s = pa.seq[si], j = pa.j[si];
  // every input is requested before anything is used: the kernel is a chain of memory round trips otherwise
  constexpr int XMAX = 8, CMAX = 16;                   // d <= 2048 and <= 4096 candidate tiles stay in registers
  float xv[XMAX], gv[XMAX], cv[CMAX];
  int ci[CMAX];
  const bool in_regs = d <= XMAX * (int)blockDim.x && pick_tiles <= CMAX * (int)blockDim.x;
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < CMAX; ++u) {
      const int t = threadIdx.x + u * blockDim.x;
      cv[u] = t < pick_tiles ? pick_val[(size_t)si * pick_tiles + t] : -INFINITY;
      ci[u] = t < pick_tiles ? pick_idx[(size_t)si * pick_tiles + t] : 0x7fffffff;
    }
#pragma unroll
    for (int u = 0; u < XMAX; ++u) {
      const int k = threadIdx.x + u * blockDim.x;
      xv[u] = k < d ? x[(size_t)si * ldx + k] : 0.f;
      gv[u] = k < d ? g[k] : 0.f;
    }
  }
  const float rs = row_scale(ssq, ssq_stride, si, inv_dim, eps);
  float* ho = hidden + (size_t)(s * G1 + j) * d;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < XMAX; ++u) {
      const int k = threadIdx.x + u * blockDim.x;
      if (k < d) ho[k] = xv[u] * gv[u] * rs;
    }
#pragma unroll
    for (int u = 0; u < CMAX; ++u)
      if (cv[u] > best || (cv[u] == best && ci[u] < bi)) { best = cv[u]; bi = ci[u]; }
  } else {
    for (int k = threadIdx.x; k < d; k += blockDim.x) ho[k] = x[(size_t)si * ldx + k] * g[k] * rs;
    for (int t = threadIdx.x; t < pick_tiles; t += blockDim.x) {
      const float v = pick_val[(size_t)si * pick_tiles + t];
      const int i = pick_idx[(size_t)si * pick_tiles + t];
      if (v > best || (v == best && i < bi)) { best = v; bi = i; }
    }
  }
  block_argmax(best, bi, redv, redi);       // (its barriers also separate the reads of x and ssq above from the writes below)
  bi = checked_token(bi, V, threadIdx.x == 0 ? host_bad : nullptr, s);   // candidates without a finite value leave the sentinel
  if (threadIdx.x == 0) draft_tok[s * G1 + j] = bi;
  if (E) embed_row_w16(E + (size_t)bi * d, d, si, next, red);
}

// pre-verification head on the un-normalised residual rows: z = (x*g*rs) . cls
// One wave per row of the block; every input of the wave (the row, the gain, both head rows, the row's sums of
// squares) is requested with 16-byte loads before the first is used: the kernel is one memory round trip, not a chain.
__global__ void mb_head_w16_kernel(const float* x, int ldx, const float* __restrict__ g, const u64* ssq,
                                   int ssq_stride, float inv_dim, float eps, const float* __restrict__ cls, int d, int b, HaltArgs ha,
                                   float* __restrict__ alpha, int* __restrict__ stop, int* __restrict__ host_stop,
                                   const uint16_t* __restrict__ E, const int* __restrict__ next_tok, EmbedOut next) {
  __shared__ float al[32];
  __shared__ float red[16];
  const int si = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = blockDim.x >> 6;
  constexpr int CH = 4;                                 // 16-byte chunks per lane held in registers: d <= 1024
  const int n4 = d >> 2;
  for (int jj = wv; jj < b; jj += nw) {
    const int r = si * b + jj;
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)r * ldx);
    const float4* g4 = reinterpret_cast<const float4*>(g);
    const float4* c0 = reinterpret_cast<const float4*>(cls);
    const float4* c1 = reinterpret_cast<const float4*>(cls + d);
    float z0 = 0.f, z1 = 0.f;
    u64 sq[SSQ_SUB];
#pragma unroll
    for (int i = 0; i < SSQ_SUB; ++i) sq[i] = ssq[(size_t)i * ssq_stride + r];
    if (n4 <= CH * 64) {
      float4 xv[CH], gv[CH], a0[CH], a1[CH];
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int k = min(lane + 64 * u, n4 - 1);        // a chunk past the end repeats the last one and is not added
        xv[u] = xr[k]; gv[u] = g4[k]; a0[u] = c0[k]; a1[u] = c1[k];
      }
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        if (lane + 64 * u < n4) {
          const float v0 = xv[u].x * gv[u].x, v1 = xv[u].y * gv[u].y, v2 = xv[u].z * gv[u].z, v3 = xv[u].w * gv[u].w;
          z0 += v0 * a0[u].x + v1 * a0[u].y + v2 * a0[u].z + v3 * a0[u].w;
          z1 += v0 * a1[u].x + v1 * a1[u].y + v2 * a1[u].z + v3 * a1[u].w;
        }
      }
    } else {
      for (int k = lane; k < n4; k += 64) {
        const float4 xv = xr[k], gv = g4[k], a0 = c0[k], a1 = c1[k];
        const float v0 = xv.x * gv.x, v1 = xv.y * gv.y, v2 = xv.z * gv.z, v3 = xv.w * gv.w;
        z0 += v0 * a0.x + v1 * a0.y + v2 * a0.z + v3 * a0.w;
        z1 += v0 * a1.x + v1 * a1.y + v2 * a1.z + v3 * a1.w;
      }
    }
    u64 t = 0;
#pragma unroll
    for (int i = 0; i < SSQ_SUB; ++i) t += sq[i];
    const float rs = 1.0f / sqrtf((float)t * SSQ_INV_SCALE * inv_dim + eps);
    z0 = wave_sum(z0) * rs;
    z1 = wave_sum(z1) * rs;
    if (lane == 0) al[jj] = 1.0f / (1.0f + expf(z0 - z1));
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int jj = 0; jj < b; ++jj) alpha[si * b + jj] = al[jj];
    const int st = ha.force[si] >= 0 ? ha.force[si] : halt_decision(al, b, ha.t[si], ha.rule);
    stop[si] = st;
    host_stop[ha.seq[si]] = ha.ticket[si] * 2 + st;
  }
  // E != null (single-sequence launches only: row 0 of next.x is one of the rows this block has just read): the
  // embedding of the newest draft token, which the next round's first draft step would start with if drafting goes on
  if (E) embed_row_w16(E + (size_t)next_tok[0] * d, d, 0, next, red);
}
