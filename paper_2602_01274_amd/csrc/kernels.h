// Device kernels of the Pacer hot path for gfx950 (CDNA4, wave64).
//
// Data layout conventions used by every kernel in this file
//   activations ........ f32 [rows][width], row major
//   packed activations . (bf16 models) f16 operand tiles for the MFMA GEMM: tile (kt, mt) holds rows
//                        mt*16..+15 and features kt*32..+31 as 16 columns of 64 bytes: row j's 32
//                        features are contiguous, MFMA lane 16*g + j reads bytes 64*j + 16*g..+15.
//                        Rows are what a launch has few of, so a GEMM wave fetches only the 64-byte
//                        columns of live rows: operand traffic is proportional to the row count.
//   packed weights ..... the model's bf16 values stored as IEEE f16 (same bytes; the matrix units take
//                        f16 pairs with f16 activations, and converting while packing instead of in
//                        every GEMM frees three vector instructions per weight pair; bf16 -> f16 is
//                        exact down to 2^-17): tile (nt, kt) holds outputs nt*16..+15 and inputs kt*32..+31 in MFMA
//                        lane order (lane 16*g + i = output i, inputs 8*g..+7), tiles ordered
//                        [nt][kt], so a wave that walks along K for one output tile reads one
//                        contiguous stream with one 1 KiB load per step.
//   KV cache ........... f32 models: [seq][layer][K|V][position][d_model].  bf16 models: IEEE f16
//                        (same bytes as bf16, 3 more mantissa bits: K after RoPE and V are O(1)
//                        quantities, so range is no concern and rounding is what matters), in the
//                        per-head tile order given in kernels_w16.h
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define PK_MAXB 16
#define ATT_MAXR 32   // rows of one sequence in one attention launch
#define ATT_TILE 64   // keys per LDS tile

// Rows of a launch: sequence si (slot in the call's list) owns rows row_off[si]..row_off[si+1]-1
// at consecutive absolute positions starting at pos0[si]; len[si] = committed tokens.
struct SeqRows {
  int n_seqs;
  int seq[PK_MAXB];
  int row_off[PK_MAXB + 1];
  int pos0[PK_MAXB];
  int len[PK_MAXB];
};

__device__ __forceinline__ int find_seq(const SeqRows& sr, int r) {
  int s = 0;
  while (s + 1 < sr.n_seqs && sr.row_off[s + 1] <= r) ++s;
  return s;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);   // round to nearest even
  return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float ld_f32(const T* p);
template <> __device__ __forceinline__ float ld_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld_f32<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st_f32(T* p, float v);
template <> __device__ __forceinline__ void st_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f32<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }
template <> __device__ __forceinline__ void st_f32<_Float16>(_Float16* p, float v) { *p = (_Float16)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Block-wide sum in a fixed order (deterministic).  red: LDS scratch of >= 16 floats.
__device__ __forceinline__ float block_sum(float v, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_max(v);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}
// Block-wide argmax; the lowest index wins among equal values.  Result valid in all threads.
__device__ __forceinline__ void block_argmax(float& v, int& idx, float* redv, int* redi) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(v, o, 64);
    int oi = __shfl_xor(idx, o, 64);
    if (ov > v || (ov == v && oi < idx)) { v = ov; idx = oi; }
  }
  __syncthreads();
  if (lane == 0) { redv[w] = v; redi[w] = idx; }
  __syncthreads();
  v = redv[0]; idx = redi[0];
  for (int i = 1; i < nw; ++i)
    if (redv[i] > v || (redv[i] == v && redi[i] < idx)) { v = redv[i]; idx = redi[i]; }
}

// ------------------------------------------------------------------ Philox-4x32-10
// Salmon et al., "Parallel random numbers: as easy as 1, 2, 3" (SC'11).
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
    c = make_uint4(hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0);
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c;
}
// uniform in (0,1), exactly representable in f32: ((bits >> 9) + 0.5) * 2^-23
__device__ __forceinline__ float u01(uint32_t bits) { return ((float)(bits >> 9) + 0.5f) * 1.1920928955078125e-07f; }
__device__ __forceinline__ float gumbel(float u) { return -logf(-logf(u)); }
#define PURPOSE_DRAFT 0u
#define PURPOSE_ACCEPT 1u
#define PURPOSE_NEXT 2u
// four uniforms for vocabulary ids 4*blk..4*blk+3
__device__ __forceinline__ uint4 vocab_bits(uint64_t seed, int seq, uint32_t step, uint32_t row, uint32_t purpose, uint32_t blk) {
  return philox4x32_10(make_uint4(blk, row, step, purpose | ((uint32_t)seq << 8)), (uint32_t)seed, (uint32_t)(seed >> 32));
}

// ------------------------------------------------------------------ token ids as table indices
// A token id that is about to be stored, or used as an index, is checked against the vocabulary first.  An argmax
// over logits that held no finite value leaves the sentinel 0x7fffffff, and a caller may hand in anything: such an
// id is replaced by the nearest valid one, so that no later load leaves its table, and the sequence's word in
// pinned host memory (host_bad, may be null) is set, which the host turns into an error at its next read-back.
__device__ __forceinline__ int checked_token(int tok, int V, int* host_bad, int seq) {
  if ((unsigned)tok < (unsigned)V) return tok;
  if (host_bad) {
    host_bad[seq] = 1;
    __threadfence_system();
  }
  return tok < 0 ? 0 : V - 1;
}
// prompt tokens into the sequence's token buffer
__global__ void copy_tokens_kernel(int* __restrict__ dst, const int* __restrict__ src, int n, int V, int* host_bad, int seq) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = checked_token(src[i], V, host_bad, seq);
}

// ------------------------------------------------------------------ embedding gather
// token of (sequence, position): committed token below len, else the draft made at that position
template <typename T>
__global__ void embed_rows_kernel(const T* __restrict__ E, const int* __restrict__ tokens, const int* __restrict__ draft_tok,
                                  SeqRows sr, int max_seq, int G1, int d, float* __restrict__ x, int ldx) {
  const int r = blockIdx.x;
  const int si = find_seq(sr, r);
  const int s = sr.seq[si];
  const int p = sr.pos0[si] + (r - sr.row_off[si]);
  const int tok = p < sr.len[si] ? tokens[(size_t)s * max_seq + p] : draft_tok[s * G1 + (p - sr.len[si])];
  const T* e = E + (size_t)tok * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) x[(size_t)r * ldx + k] = ld_f32<T>(e + k);
}

// input rows of the pre-verification layer: hidden + PosEmb[e] (e = 0 for prefix rows)
struct MbRows { int src_row0[PK_MAXB]; int e0[PK_MAXB]; };
__global__ void mb_input_kernel(const float* __restrict__ src, int lds, const float* __restrict__ posemb, SeqRows sr, MbRows mr,
                                int d, float* __restrict__ x, int ldx) {
  const int r = blockIdx.x;
  const int si = find_seq(sr, r);
  const int rr = r - sr.row_off[si];
  const float* h = src + (size_t)(mr.src_row0[si] + rr) * lds;
  const float* e = posemb + (size_t)(mr.e0[si] < 0 ? 0 : mr.e0[si] + rr) * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) x[(size_t)r * ldx + k] = h[k] + e[k];
}

// ------------------------------------------------------------------ f32 path: norm and activation
// RMSNorm of R rows (one block each); writes the normalised rows as f32 (xn) and optionally scattered
// copies for the draft's hidden-state ring (hid_out row = seq*G1 + draft index).
__global__ void rmsnorm_pack_kernel(const float* __restrict__ x, int ldx, const float* __restrict__ g, float eps, int R, int d,
                                    float* __restrict__ xn, int ldxn, float* __restrict__ hid_out, int G1, SeqRows sr) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  const int ng = d >> 3;
  if (r >= R) return;
  const float* xr = x + (size_t)r * ldx;
  float ss = 0.f;
  for (int k = threadIdx.x; k < d; k += blockDim.x) { const float v = xr[k]; ss += v * v; }
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  float* ho = nullptr;
  if (hid_out) {
    const int si = find_seq(sr, r);
    const int j = sr.pos0[si] + (r - sr.row_off[si]) - (sr.len[si] - 1);
    ho = hid_out + (size_t)(sr.seq[si] * G1 + j) * d;
  }
  for (int kg = threadIdx.x; kg < ng; kg += blockDim.x) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = xr[kg * 8 + i] * inv * g[kg * 8 + i];
#pragma unroll
    for (int i = 0; i < 8; ++i) xn[(size_t)r * ldxn + kg * 8 + i] = v[i];
    if (ho) {
#pragma unroll
      for (int i = 0; i < 8; ++i) ho[kg * 8 + i] = v[i];
    }
  }
}

// SwiGLU: act = silu(gate) * up for gu = [gate | up] rows, f32
__global__ void swiglu_pack_kernel(const float* __restrict__ gu, int ldg, int R, int F, float* __restrict__ act, int lda) {
  const int r = blockIdx.y;
  const int kg = blockIdx.x * blockDim.x + threadIdx.x;
  if (kg >= (F >> 3) || r >= R) return;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float gt = gu[(size_t)r * ldg + kg * 8 + i], up = gu[(size_t)r * ldg + F + kg * 8 + i];
    act[(size_t)r * lda + kg * 8 + i] = gt / (1.0f + expf(-gt)) * up;
  }
}

// ------------------------------------------------------------------ output row mapping of a GEMM
#define ROWMAP_ID 0      // out row = r
#define ROWMAP_RING 1    // out row = seq*G1 + draft index      (draft logits ring)
#define ROWMAP_LIST 2    // out row = slot*G1 + row within seq  (verify logits)
__device__ __forceinline__ int map_row(const SeqRows& sr, int mode, int G1, int r) {
  if (mode == ROWMAP_ID) return r;
  const int si = find_seq(sr, r);
  const int rr = r - sr.row_off[si];
  if (mode == ROWMAP_LIST) return si * G1 + rr;
  return sr.seq[si] * G1 + (sr.pos0[si] + rr - (sr.len[si] - 1));
}

// bf16 -> f16 of 8 weights (exact for |w| >= 2^-17; smaller ones round to the nearest f16 subnormal,
// absolute error <= 2^-25).  Done once, when a matrix is packed.
__device__ __forceinline__ u32x4 bf16x8_to_f16x8(u32x4 w) {
  half8 h;
  const uint32_t u[4] = {w[0], w[1], w[2], w[3]};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(u[i] << 16), hi = __uint_as_float(u[i] & 0xffff0000u);
    h[2 * i] = (_Float16)lo;
    h[2 * i + 1] = (_Float16)hi;
  }
  return __builtin_bit_cast(u32x4, h);
}

// Plain f32 GEMM for f32 models and tiny heads: one wave per output feature, rows in groups of 8.
__global__ void gemm_f32_kernel(const float* __restrict__ W, const float* __restrict__ X, int ldx, float* __restrict__ out, int ldo,
                                int R, int N, int K, int accumulate, SeqRows sr, int rowmap, int G1) {
  const int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (n >= N) return;
  const float* w = W + (size_t)n * K;
  for (int r0 = 0; r0 < R; r0 += 8) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int k = lane; k < K; k += 64) {
      const float wv = w[k];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (r0 + i < R) acc[i] += wv * X[(size_t)(r0 + i) * ldx + k];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float s = wave_sum(acc[i]);
      if (lane == 0 && r0 + i < R) {
        float* o = out + (size_t)map_row(sr, rowmap, G1, r0 + i) * ldo + n;
        *o = accumulate ? *o + s : s;
      }
    }
  }
}

// ------------------------------------------------------------------ RoPE
// cos/sin table [R][hd/2][2] for this launch's absolute positions, evaluated in double
__global__ void rope_table_kernel(SeqRows sr, int hd, float theta, float* __restrict__ tab) {
  const int r = blockIdx.x, j = threadIdx.x;
  const int half = hd >> 1;
  if (j >= half) return;
  const int si = find_seq(sr, r);
  const double pos = (double)(sr.pos0[si] + (r - sr.row_off[si]));
  const double inv = pow((double)theta, -2.0 * (double)j / (double)hd);
  double sn, cs;
  sincos(pos * inv, &sn, &cs);
  tab[((size_t)r * half + j) * 2] = (float)cs;
  tab[((size_t)r * half + j) * 2 + 1] = (float)sn;
}

// rotate q in place, rotate k and copy v into the KV cache (rotate-half pairing j, j+hd/2)
template <typename KVT>
__global__ void rope_append_kernel(float* __restrict__ qkv, int ld, const float* __restrict__ tab, SeqRows sr, int d, int hd,
                                   KVT* __restrict__ kv, int layer, int n_layers, int max_seq, int kv_only) {
  const int r = blockIdx.x, h = blockIdx.y, j = threadIdx.x;
  const int half = hd >> 1;
  if (j >= half) return;
  const int si = find_seq(sr, r);
  const int pos = sr.pos0[si] + (r - sr.row_off[si]);
  const float cs = tab[((size_t)r * half + j) * 2], sn = tab[((size_t)r * half + j) * 2 + 1];
  float* row = qkv + (size_t)r * ld;
  const int c0 = h * hd + j, c1 = c0 + half;
  if (!kv_only) {
    const float a = row[c0], b = row[c1];
    row[c0] = a * cs - b * sn;
    row[c1] = b * cs + a * sn;
  }
  KVT* K = kv + (((size_t)sr.seq[si] * n_layers + layer) * 2) * (size_t)max_seq * d + (size_t)pos * d;
  KVT* V = K + (size_t)max_seq * d;
  const float a = row[d + c0], b = row[d + c1];
  st_f32<KVT>(K + c0, a * cs - b * sn);
  st_f32<KVT>(K + c1, b * cs + a * sn);
  st_f32<KVT>(V + c0, row[2 * d + c0]);
  st_f32<KVT>(V + c1, row[2 * d + c1]);
}

// ------------------------------------------------------------------ attention over the KV cache
// One block = (chunk of key tiles, head, sequence).  All rows of the sequence (<= 32) share every
// K/V tile, which is staged once in LDS.  Row r attends to keys 0..pos_r.  Online softmax over the
// tiles of the chunk; the chunk's (max, sum, weighted values) go to `part` for attn_combine.
template <typename KVT> struct KvWords;
template <> struct KvWords<float> { static constexpr int per_word = 1; };
template <> struct KvWords<_Float16> { static constexpr int per_word = 2; };
__device__ __forceinline__ float f16lo(uint32_t w) { return (float)__builtin_bit_cast(half2v, w)[0]; }
__device__ __forceinline__ float f16hi(uint32_t w) { return (float)__builtin_bit_cast(half2v, w)[1]; }
template <typename KVT> __device__ __forceinline__ float kv_dim(const uint32_t* row, int dim);
template <> __device__ __forceinline__ float kv_dim<float>(const uint32_t* row, int dim) { return __uint_as_float(row[dim]); }
template <> __device__ __forceinline__ float kv_dim<_Float16>(const uint32_t* row, int dim) {
  const uint32_t w = row[dim >> 1];
  return (dim & 1) ? f16hi(w) : f16lo(w);
}

template <typename KVT, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(const float* __restrict__ q, int ldq, const KVT* __restrict__ kv, int layer,
                                                           int n_layers, int max_seq, int d, SeqRows sr, int tiles_per_chunk,
                                                           int n_chunks, int H, float* __restrict__ part) {
  constexpr int WORDS = HD / KvWords<KVT>::per_word;   // 32-bit words per key row of one head
  constexpr int STR = WORDS + 1;                        // odd stride: conflict-free column access
  constexpr int DPL = HD / 64;                          // output dims per lane
  __shared__ float Qs[ATT_MAXR][HD];
  __shared__ uint32_t Kt[ATT_TILE * STR];
  __shared__ uint32_t Vt[ATT_TILE * STR];
  __shared__ float S[ATT_MAXR][ATT_TILE];
  __shared__ float sm[ATT_MAXR], sl[ATT_MAXR], sc[ATT_MAXR];

  const int chunk = blockIdx.x, h = blockIdx.y, si = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int r0 = sr.row_off[si], Rs = sr.row_off[si + 1] - r0;
  const int pos0 = sr.pos0[si];
  const int n_keys = pos0 + Rs;                          // keys visible to the last row
  const int n_tiles = (n_keys + ATT_TILE - 1) / ATT_TILE;
  const int t_begin = chunk * tiles_per_chunk, t_end = min(n_tiles, t_begin + tiles_per_chunk);
  const float scale = 1.0f / sqrtf((float)HD);
  const KVT* Kb = kv + (((size_t)sr.seq[si] * n_layers + layer) * 2) * (size_t)max_seq * d + h * HD;
  const KVT* Vb = Kb + (size_t)max_seq * d;

  for (int i = tid; i < Rs * HD; i += 256) Qs[i / HD][i % HD] = q[(size_t)(r0 + i / HD) * ldq + h * HD + (i % HD)] * scale;
  if (tid < ATT_MAXR) { sm[tid] = -INFINITY; sl[tid] = 0.f; sc[tid] = 1.f; }
  float acc[ATT_MAXR / 4][DPL];
#pragma unroll
  for (int i = 0; i < ATT_MAXR / 4; ++i)
#pragma unroll
    for (int e = 0; e < DPL; ++e) acc[i][e] = 0.f;
  __syncthreads();

  for (int t = t_begin; t < t_end; ++t) {
    const int key0 = t * ATT_TILE;
    // stage K and V tiles: 16-byte global reads, 4-byte LDS writes
    constexpr int V4 = WORDS / 4;                       // uint4 per key
    for (int i = tid; i < ATT_TILE * V4; i += 256) {
      const int key = i / V4, c = i % V4;
      uint4 kq = make_uint4(0, 0, 0, 0), vq = kq;
      if (key0 + key < n_keys) {
        kq = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(Kb + (size_t)(key0 + key) * d) + c * 4);
        vq = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(Vb + (size_t)(key0 + key) * d) + c * 4);
      }
      uint32_t* kd = Kt + key * STR + c * 4;
      uint32_t* vd = Vt + key * STR + c * 4;
      kd[0] = kq.x; kd[1] = kq.y; kd[2] = kq.z; kd[3] = kq.w;
      vd[0] = vq.x; vd[1] = vq.y; vd[2] = vq.z; vd[3] = vq.w;
    }
    __syncthreads();
    // scores: thread = (key, row group)
    {
      float s[ATT_MAXR / 4];
#pragma unroll
      for (int i = 0; i < ATT_MAXR / 4; ++i) s[i] = 0.f;
      const uint32_t* krow = Kt + lane * STR;
      for (int w = 0; w < WORDS; ++w) {
        const uint32_t kw = krow[w];
        if (KvWords<KVT>::per_word == 2) {
          const float k0 = f16lo(kw), k1 = f16hi(kw);
#pragma unroll
          for (int i = 0; i < ATT_MAXR / 4; ++i) {
            const int r = wv + 4 * i;
            if (r < Rs) s[i] += Qs[r][2 * w] * k0 + Qs[r][2 * w + 1] * k1;
          }
        } else {
          const float k0 = __uint_as_float(kw);
#pragma unroll
          for (int i = 0; i < ATT_MAXR / 4; ++i) {
            const int r = wv + 4 * i;
            if (r < Rs) s[i] += Qs[r][w] * k0;
          }
        }
      }
#pragma unroll
      for (int i = 0; i < ATT_MAXR / 4; ++i) {
        const int r = wv + 4 * i;
        if (r < Rs) S[r][lane] = (key0 + lane <= pos0 + r) ? s[i] : -INFINITY;
      }
    }
    __syncthreads();
    // online softmax: wave wv owns rows wv, wv+4, ...; lane = key
    for (int r = wv; r < Rs; r += 4) {
      const float sv = S[r][lane];
      const float mo = sm[r];
      const float mn = fmaxf(mo, wave_max(sv));
      const float p = (mn == -INFINITY) ? 0.f : expf(sv - mn);
      const float ps = wave_sum(p);
      S[r][lane] = p;
      if (lane == 0) {
        const float corr = (mo == -INFINITY) ? 1.f : expf(mo - mn);
        sc[r] = corr;
        sl[r] = sl[r] * corr + ps;
        sm[r] = mn;
      }
    }
    __syncthreads();
    // weighted values: thread = (dims lane*DPL.., row group)
#pragma unroll
    for (int i = 0; i < ATT_MAXR / 4; ++i) {
      const int r = wv + 4 * i;
      if (r < Rs) {
        const float c = sc[r];
#pragma unroll
        for (int e = 0; e < DPL; ++e) acc[i][e] *= c;
      }
    }
    for (int key = 0; key < ATT_TILE; ++key) {
      float vv[DPL];
#pragma unroll
      for (int e = 0; e < DPL; ++e) vv[e] = kv_dim<KVT>(Vt + key * STR, lane * DPL + e);
#pragma unroll
      for (int i = 0; i < ATT_MAXR / 4; ++i) {
        const int r = wv + 4 * i;
        if (r < Rs) {
          const float p = S[r][key];
#pragma unroll
          for (int e = 0; e < DPL; ++e) acc[i][e] += p * vv[e];
        }
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < ATT_MAXR / 4; ++i) {
    const int r = wv + 4 * i;
    if (r < Rs) {
      float* o = part + (((size_t)(r0 + r) * H + h) * n_chunks + chunk) * (HD + 2);
#pragma unroll
      for (int e = 0; e < DPL; ++e) o[lane * DPL + e] = acc[i][e];
      if (lane == 0) { o[HD] = sm[r]; o[HD + 1] = sl[r]; }
    }
  }
}

// merge the chunks' partial softmaxes: grid (rows, heads), block HD threads
__global__ void attn_combine_kernel(const float* __restrict__ part, int n_chunks, int H, int HD, float* __restrict__ out, int ldo) {
  const int r = blockIdx.x, h = blockIdx.y, dim = threadIdx.x;
  const float* p = part + ((size_t)r * H + h) * n_chunks * (HD + 2);
  float M = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, p[(size_t)c * (HD + 2) + HD]);
  float L = 0.f, a = 0.f;
  for (int c = 0; c < n_chunks; ++c) {
    const float m = p[(size_t)c * (HD + 2) + HD];
    if (m == -INFINITY) continue;
    const float w = expf(m - M);
    L += p[(size_t)c * (HD + 2) + HD + 1] * w;
    a += p[(size_t)c * (HD + 2) + dim] * w;
  }
  out[(size_t)r * ldo + h * HD + dim] = a / L;
}

// ------------------------------------------------------------------ token choice of the draft model
// one block per listed sequence: y = argmax(logits) or Gumbel-max sample; row j of the ring
struct PickArgs { int n_seqs; int seq[PK_MAXB]; int j[PK_MAXB]; };
__global__ __launch_bounds__(1024) void pick_token_kernel(const float* __restrict__ ring, int* __restrict__ draft_tok, PickArgs pa,
                                                          int G1, int V, int mode, uint64_t seed, uint32_t step, int* host_bad) {
  __shared__ float redv[16];
  __shared__ int redi[16];
  const int si = blockIdx.x, s = pa.seq[si], j = pa.j[si];
  const float* lg = ring + (size_t)(s * G1 + j) * V;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int blk = threadIdx.x; blk * 4 < V; blk += blockDim.x) {
    float g4[4] = {0.f, 0.f, 0.f, 0.f};
    if (mode) {
      const uint4 b = vocab_bits(seed, s, step, (uint32_t)(j + 1), PURPOSE_DRAFT, (uint32_t)blk);
      g4[0] = gumbel(u01(b.x)); g4[1] = gumbel(u01(b.y)); g4[2] = gumbel(u01(b.z)); g4[3] = gumbel(u01(b.w));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int v = blk * 4 + e;
      if (v < V) {
        const float val = lg[v] + g4[e];
        if (val > best) { best = val; bi = v; }
      }
    }
  }
  block_argmax(best, bi, redv, redi);
  if (threadIdx.x == 0) draft_tok[s * G1 + j] = checked_token(bi, V, host_bad, s);
}

// ------------------------------------------------------------------ pre-verification head + halting test
// xn: final-norm output of M_B, rows grouped per sequence (b rows each).  alpha_j = softmax(z)[1]
// = 1/(1+exp(z0-z1)); stop = (mean alpha <= t) with the mean summed in index order in f32.
// rule: 0 mean, 1 any, 2 last.  seq/ticket: the stop flag also goes to pinned host memory as
// host_stop[seq] = ticket*2 + stop, which the host polls instead of synchronising the stream.
// force: -1 = decide by the rule; 0 / 1 = the flag is forced (test tap: sweeps over stop patterns), the kernel still
// computes and writes alpha
struct HaltArgs { int n_seqs; int rule; float t[PK_MAXB]; int seq[PK_MAXB]; int ticket[PK_MAXB]; int force[PK_MAXB]; };
// the halting test of one block, decided in f32 (al: the block's alpha values in index order)
__device__ __forceinline__ int halt_decision(const float* al, int b, float t, int rule) {
  if (rule == 1) {
    int any = 0;
    for (int j = 0; j < b; ++j) any |= (al[j] <= t) ? 1 : 0;
    return any;
  }
  if (rule == 2) return (al[b - 1] <= t) ? 1 : 0;
  float s = 0.f;
  for (int j = 0; j < b; ++j) s += al[j];
  return (s / (float)b <= t) ? 1 : 0;
}
__global__ void mb_head_kernel(const float* __restrict__ xn, int ldx, const float* __restrict__ cls, int d, int b, HaltArgs ha,
                               float* __restrict__ alpha, int* __restrict__ stop, int* __restrict__ host_stop) {
  __shared__ float al[32];
  const int si = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (int j = wv; j < b; j += nw) {
    const float* x = xn + (size_t)(si * b + j) * ldx;
    float z0 = 0.f, z1 = 0.f;
    for (int k = lane; k < d; k += 64) { z0 += x[k] * cls[k]; z1 += x[k] * cls[d + k]; }
    z0 = wave_sum(z0); z1 = wave_sum(z1);
    if (lane == 0) al[j] = 1.0f / (1.0f + expf(z0 - z1));
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int j = 0; j < b; ++j) alpha[si * b + j] = al[j];
    const int st = ha.force[si] >= 0 ? ha.force[si] : halt_decision(al, b, ha.t[si], ha.rule);
    stop[si] = st;
    host_stop[ha.seq[si]] = ha.ticket[si] * 2 + st;
  }
}

// ------------------------------------------------------------------ acceptance (Eq. 5)
// slot: the sequence's index in the verify call that wrote the logits (row slot*G1 + i of tl, entry slot of the
// caller's n / z arrays).  The kernels run in two phases: phase 0 covers rows i < gamma (everything a step needs
// unless every draft is accepted), phase 1 the bonus row i = gamma of the sequences that accepted all drafts.
// qslot: the sequence's block of G1 rows in the draft logits and draft token buffers (the sequence id for a context's
// rings); seq itself keys the random streams and indexes the committed tokens and the host words.
struct AccArgs { int n_seqs; int seq[PK_MAXB]; int slot[PK_MAXB]; int qslot[PK_MAXB]; int gamma[PK_MAXB]; int len[PK_MAXB]; float beta[PK_MAXB]; };

// One row of logits is split into ACC_CHUNKS vocabulary ranges, one block each (a single block per row
// spent 53 us walking 32000 entries three times).  Three launches:
//   accept_stats_kernel   per (row, chunk): running max and sum of exp of the effective target logits and
//                         of the draft logits over the chunk                                  (sampling only)
//   accept_rows_kernel    per (row, chunk): log-sum-exp of the row from the chunk statistics (fixed chunk
//                         order, so every chunk of a row derives the same value), then the chunk's best
//                         candidates; chunk 0 also takes the row's accept test
//   accept_finalize_kernel per sequence: best candidate over the chunks of each row, first rejection, tokens
// Rows i < gamma first; the bonus row i = gamma (whose draft logits cost one more draft forward) only for the
// sequences that turn out to have accepted every draft.
#define ACC_CHUNKS 16
#define ACC_PART 8      // floats per (row, chunk): [0..3] = mp, sp, mq, sq ; [4..7] = best, bi, bestp, bip

__device__ __forceinline__ void acc_chunk_range(int V, int chunk, int& v0, int& v1) {
  const int per = ((V + ACC_CHUNKS - 1) / ACC_CHUNKS + 3) & ~3;   // multiple of 4: a Philox block never straddles chunks
  v0 = min(V, chunk * per);
  v1 = min(V, v0 + per);
}

// grid (gamma_max+1, n_seqs, ACC_CHUNKS)
// done_z (phase 1 only, may be null): the phase-0 results; a sequence whose entry is >= 0 already has its token
// (a draft was rejected) and the bonus row is skipped.
__global__ __launch_bounds__(256) void accept_stats_kernel(const float* __restrict__ tl, const float* __restrict__ ring, AccArgs aa, int G1,
                                                           int V, int phase, float* __restrict__ part, const int* __restrict__ done_z) {
  __shared__ float redv[16];
  const int si = blockIdx.y, ch = blockIdx.z, sl = aa.slot[si];
  const int i = phase ? aa.gamma[si] : blockIdx.x;
  if (!phase && i >= aa.gamma[si]) return;
  if (phase && done_z && done_z[sl] >= 0) return;
  const float beta = aa.beta[si];
  const float* t = tl + (size_t)(sl * G1 + i) * V;
  const float* q = ring + (size_t)(aa.qslot[si] * G1 + i) * V;
  int v0, v1;
  acc_chunk_range(V, ch, v0, v1);
  float mp = -INFINITY, mq = -INFINITY;
  for (int v = v0 + threadIdx.x; v < v1; v += blockDim.x) { mp = fmaxf(mp, t[v] + beta * q[v]); mq = fmaxf(mq, q[v]); }
  mp = block_max(mp, redv);
  mq = block_max(mq, redv);
  float sp = 0.f, sq = 0.f;
  for (int v = v0 + threadIdx.x; v < v1; v += blockDim.x) { sp += expf(t[v] + beta * q[v] - mp); sq += expf(q[v] - mq); }
  sp = block_sum(sp, redv);
  sq = block_sum(sq, redv);
  if (threadIdx.x == 0) {
    float* o = part + ((size_t)(sl * G1 + i) * ACC_CHUNKS + ch) * ACC_PART;
    o[0] = mp; o[1] = sp; o[2] = mq; o[3] = sq;
  }
}

// grid (gamma_max+1, n_seqs, ACC_CHUNKS): row i of sequence slot si, vocabulary chunk ch.  Writes the chunk's
// candidates (token emitted if this row is where drafting is cut) and, from chunk 0, rej (row's draft rejected).
__global__ __launch_bounds__(256) void accept_rows_kernel(const float* __restrict__ tl, const float* __restrict__ ring,
                                                          const int* __restrict__ draft_tok, AccArgs aa, int G1, int V, int mode,
                                                          uint64_t seed, uint32_t step, int phase, float* __restrict__ part,
                                                          int* __restrict__ rej, const int* __restrict__ done_z) {
  __shared__ float redv[16];
  __shared__ int redi[16];
  const int si = blockIdx.y, ch = blockIdx.z, s = aa.seq[si], sl = aa.slot[si];
  const int gamma = aa.gamma[si];
  const int i = phase ? gamma : blockIdx.x;
  if (!phase && i >= gamma) return;
  if (phase && done_z && done_z[sl] >= 0) return;
  const float beta = aa.beta[si];
  const float* t = tl + (size_t)(sl * G1 + i) * V;
  const float* q = ring + (size_t)(aa.qslot[si] * G1 + i) * V;
  const int y = i < gamma ? draft_tok[aa.qslot[si] * G1 + i] : -1;
  float* prow = part + (size_t)(sl * G1 + i) * ACC_CHUNKS * ACC_PART;
  float* o = prow + ch * ACC_PART;
  int v0, v1;
  acc_chunk_range(V, ch, v0, v1);
  if (mode == 0) {
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int v = v0 + threadIdx.x; v < v1; v += blockDim.x) {
      const float e = t[v] + beta * q[v];
      if (e > best) { best = e; bi = v; }
    }
    block_argmax(best, bi, redv, redi);
    if (threadIdx.x == 0) {
      o[4] = -INFINITY; o[5] = __int_as_float(0x7fffffff);
      o[6] = best; o[7] = __int_as_float(bi);
    }
    return;
  }
  // log-sum-exp of effective target and of draft logits from the chunk statistics
  float mp = -INFINITY, mq = -INFINITY;
  for (int c = 0; c < ACC_CHUNKS; ++c) { mp = fmaxf(mp, prow[c * ACC_PART]); mq = fmaxf(mq, prow[c * ACC_PART + 2]); }
  float sp = 0.f, sq = 0.f;
  for (int c = 0; c < ACC_CHUNKS; ++c) {
    const float m1 = prow[c * ACC_PART], m2 = prow[c * ACC_PART + 2];
    if (m1 > -INFINITY) sp += prow[c * ACC_PART + 1] * expf(m1 - mp);
    if (m2 > -INFINITY) sq += prow[c * ACC_PART + 3] * expf(m2 - mq);
  }
  const float lsp = mp + logf(sp), lsq = mq + logf(sq);
  // candidate token: Gumbel-max over log max(0, p - q) (rows < gamma) or log p (bonus row);
  // if no residual mass exists the row falls back to log p with the same noise
  float best = -INFINITY, bestp = -INFINITY;
  int bi = 0x7fffffff, bip = 0x7fffffff;
  for (int blk = (v0 >> 2) + threadIdx.x; blk * 4 < v1; blk += blockDim.x) {
    const uint4 b = vocab_bits(seed, s, step, (uint32_t)(i + 1), PURPOSE_NEXT, (uint32_t)blk);
    const float g4[4] = {gumbel(u01(b.x)), gumbel(u01(b.y)), gumbel(u01(b.z)), gumbel(u01(b.w))};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int v = blk * 4 + e;
      if (v < v1) {
        const float lp = t[v] + beta * q[v] - lsp;
        const float kp = lp + g4[e];
        if (kp > bestp) { bestp = kp; bip = v; }
        if (i < gamma) {
          const float w = expf(lp) - expf(q[v] - lsq);
          if (w > 0.f) {
            const float kr = logf(w) + g4[e];
            if (kr > best) { best = kr; bi = v; }
          }
        }
      }
    }
  }
  block_argmax(bestp, bip, redv, redi);
  if (i < gamma) block_argmax(best, bi, redv, redi);
  if (threadIdx.x == 0) {
    o[4] = best; o[5] = __int_as_float(bi);
    o[6] = bestp; o[7] = __int_as_float(bip);
    if (ch == 0) {
      int rj = 0;
      if (i < gamma) {
        const int yc = min(max(y, 0), V - 1);          // a caller-held draft id outside the vocabulary must not index past the row
        const float ratio = expf((t[yc] + beta * q[yc] - lsp) - (q[yc] - lsq));
        const uint4 b = vocab_bits(seed, s, step, (uint32_t)(i + 1), PURPOSE_ACCEPT, 0u);
        rj = (u01(b.x) > ratio) ? 1 : 0;
      }
      rej[sl * G1 + i] = rj;
    }
  }
}

// Phase 0: n = first rejected row (or gamma).  n < gamma: next token = row n's candidate, tokens appended, results
// (n, z) to the caller's arrays and to pinned host memory.  n = gamma: the bonus row has not been evaluated yet
// (its draft logits need one more draft forward): the drafts are appended and (gamma, -1) says that phase 1, which
// takes the token of row gamma, is still to come.  The ticket is written last; the host polls for it.
// skip_done (phase 1): leave a sequence alone whose phase-0 result already holds a token (out_z >= 0).
// tokens and the host words may be null (acceptance on caller-held logits without a context).
__global__ void accept_finalize_kernel(const float* __restrict__ part, const int* __restrict__ rej, const int* __restrict__ draft_tok,
                                       AccArgs aa, int G1, int mode, int phase, int max_seq, int* __restrict__ tokens,
                                       int* __restrict__ out_n, int* __restrict__ out_z, int* __restrict__ host_res,
                                       int* __restrict__ host_tick, int ticket, int skip_done, int V, int* host_bad) {
  const int si = blockIdx.x, s = aa.seq[si], sl = aa.slot[si], qs = aa.qslot[si];
  const int gamma = aa.gamma[si];
  if (phase && skip_done && out_z[sl] >= 0) return;
  int n = gamma;
  if (!phase) {
    if (mode == 0) {
      // greedy: row i's draft is rejected when it differs from the row's argmax
      for (int i = gamma - 1; i >= 0; --i) {
        const float* pr = part + (size_t)(sl * G1 + i) * ACC_CHUNKS * ACC_PART;
        float best = -INFINITY;
        int bi = 0x7fffffff;
        for (int c = 0; c < ACC_CHUNKS; ++c) {
          const float v = pr[c * ACC_PART + 6];
          const int id = __float_as_int(pr[c * ACC_PART + 7]);
          if (v > best || (v == best && id < bi)) { best = v; bi = id; }
        }
        if (bi != draft_tok[qs * G1 + i]) n = i;
      }
    } else {
      for (int i = gamma - 1; i >= 0; --i)
        if (rej[sl * G1 + i]) n = i;
    }
  }
  int z = -1;
  if (phase || n < gamma) {
    // the emitted token: best residual candidate of row n over the chunks, else best candidate of p
    const float* pr = part + (size_t)(sl * G1 + n) * ACC_CHUNKS * ACC_PART;
    float best = -INFINITY, bestp = -INFINITY;
    int bi = 0x7fffffff, bip = 0x7fffffff;
    for (int c = 0; c < ACC_CHUNKS; ++c) {
      const float v = pr[c * ACC_PART + 4], vp = pr[c * ACC_PART + 6];
      const int id = __float_as_int(pr[c * ACC_PART + 5]), idp = __float_as_int(pr[c * ACC_PART + 7]);
      if (v > best || (v == best && id < bi)) { best = v; bi = id; }
      if (vp > bestp || (vp == bestp && idp < bip)) { bestp = vp; bip = idp; }
    }
    z = (n < gamma && best > -INFINITY) ? bi : bip;
  }
  int* tk = tokens ? tokens + (size_t)s * max_seq + aa.len[si] : nullptr;
  if (!phase && tk)
    for (int k = threadIdx.x; k < n; k += blockDim.x) tk[k] = draft_tok[qs * G1 + k];
  if (threadIdx.x == 0) {
    if (z >= 0 && tk) tk[n] = checked_token(z, V, host_bad, s);   // out_z keeps the raw value: 0x7fffffff = no finite logit decided
    out_n[sl] = n;
    out_z[sl] = z;
    if (host_res) {
      host_res[2 * s] = n;
      host_res[2 * s + 1] = z;
      __threadfence_system();            // the results first, then the ticket the host polls for
      host_tick[s] = ticket;
    }
  }
}

__global__ void copy_i32_kernel(int* __restrict__ dst, const int* __restrict__ src, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = src[i];
}

// ------------------------------------------------------------------ streaming-read probe (benchmarks)
// Reads n16 16-byte words once (grid-stride, eight loads in flight per lane) and folds them into one word per
// block: what a kernel that only streams from HBM through the L1s reaches on this GPU, the practical ceiling the
// weight-streaming GEMMs are measured against.  Launched as 256 blocks of 4 waves (one wave per SIMD): of the
// shapes tried (256..8192 blocks, 4..16 loads in flight, per-wave contiguous ranges or grid-stride) that one read
// fastest, 7.0 to 7.2 TB/s on 2 GiB.
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) acc ^= src[i];
  uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o, 64);
  if ((threadIdx.x & 63) == 0) sink[(blockIdx.x * 4 + (threadIdx.x >> 6)) & 63] = x;   // keeps the loads alive; the value is not used
}
