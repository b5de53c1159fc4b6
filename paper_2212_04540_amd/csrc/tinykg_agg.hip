// Attentive knowledge-graph aggregation layer, forward and backward, for gfx950.
//
// The layer is the KG-Layer of Sec. 3.2 (Eq. 1) in the three-stage form of
// Eq. (2) -- sparse aggregation, dense map, activation -- with KGAT's attention
// as the sparse operator; the formulas are stated in include/tinykg.h.  The
// backward pass evaluates the layer's vector-Jacobian product at the SAVED
// context (Sec. 3.3, Fig. 1): every gather of a saved row unpacks and
// dequantises it on the fly (Eq. 4), no fp32 copy of E_hat or H_hat is ever
// materialised.
//
// Kernels
//   score kernels     relation-bucketed tiles: a = W_r e_t, b = W_r e_h + e_r, s = a . tanh(b);
//                     the products run on the bf16 matrix cores with every fp32 operand split
//                     exactly into three bfloat16 pieces (six piece products, fp32 accuracy)
//   attend_fwd_kernel per head: softmax over its out-edges, H_h = e_h + sum pi e_t
//   dense_fwd_kernel  J = H W^T (six piece products), E' = LeakyReLU(J), 1-bit sign mask
//   dense_bwd_kernel  grad_J from the mask, grad_H = grad_J W, grad_W = grad_J^T H_hat
//                     (dense_bwd_code_kernel: the same on saved codes, d_in = d_out = 128)
//   attend_bwd_kernel per head: pi, g_j = grad_H_h . e_hat_t, grad_s_j
//   edge kernels      relation-bucketed tiles: recompute a, b; grad_a, grad_b;
//                     W_r^T grad_a / W_r^T grad_b rows scattered to tails / heads;
//                     grad_W_r, grad_e_r accumulated per span or chunk.  Four forms:
//                     edge_code_kernel (d <= 64) and edge_coop_code_kernel (d = 128) work on the
//                     saved integer codes when a row has one (Z, scale) pair -- Eq. (4) is linear,
//                     so nothing is dequantised and every product runs on the bf16 matrix cores;
//                     edge_wave_kernel (d <= 64) and edge_bwd_kernel (d = 128) serve the other contexts
//   uniform_tail_kernel  the transposed sparse product of the uniform layer, edges in tail order
//   epilogue_kernel   fixed-order sums of the per-chunk / per-workgroup partial parameter
//                     gradients, and the heavy nodes' double-precision rows, in one launch
//
// MFMA operand convention used throughout: one 32x32 output block is
// acc[m][n] += sum_k A(m,k) B(k,n); lane l feeds row/column l%32 and the k-half
// l/32.  The contraction index is permuted so that half 0 walks k = 0..K/2-1 and
// half 1 walks k = K/2..K-1: an operand stored with k contiguous is then read
// with 128-bit LDS loads.  Rows are padded by 4 floats, which makes both the
// 128-bit row reads and the 32-bit column reads bank-conflict free.
#include "tinykg_fetch.h"
#include "tinykg_graph.h"

#include <hip/hip_runtime.h>

namespace tinykg {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int KCONT = 0;   // operand X(row, k) stored at X[row * ld + k]
constexpr int KMAJOR = 1;  // operand X(row, k) stored at X[k * ld + row]

extern __shared__ __align__(16) unsigned char smem_raw[];

__device__ __forceinline__ int acc_row(int v, int lane) {
  // row of accumulator register v inside a 32x32 MFMA block
  return (v & 3) + 4 * (lane >> 5) + 8 * (v >> 2);
}

// tanh without branches: 1 - 2 / (exp(2x) + 1) on the hardware exp2 / rcp units.  The
// subtraction from 1 bounds the ABSOLUTE error by that of the quotient (below 2e-7 for every
// x); exp overflow gives exactly 1, underflow exactly -1.  Enough for the scores
// s = a . tanh(b), whose error enters the softmax weights as an absolute error of s.
__device__ __forceinline__ float fast_tanh(float x) {
  const float e = __builtin_amdgcn_exp2f(x * 2.885390081777927f);   // exp(2x)
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
}

// tanh accurate in RELATIVE terms, for grad_a = grad_s tanh(b), which inherits the relative
// error of tanh: near 0 the form above loses the value's leading digits in the subtraction.
// |x| < 1/8: the odd series x - x^3/3 + 2x^5/15 (truncation below 3e-7 of the value);
// elsewhere the form above, whose absolute error is then below 2e-6 of the value.
__device__ __forceinline__ float tanh_rel(float x) {
  const float x2 = x * x;
  const float small = fmaf(x * x2, fmaf(x2, 2.0f / 15.0f, -1.0f / 3.0f), x);
  return fabsf(x) < 0.125f ? small : fast_tanh(x);
}

template <int AM, int BM>
__device__ __forceinline__ void mfma_block(const float* __restrict__ A, int lda,
                                           const float* __restrict__ B, int ldb, int K,
                                           floatx16& acc) {
  const int lane = threadIdx.x & 63, r = lane & 31, hh = lane >> 5;
  const int KH = K >> 1;
  const float* ap = (AM == KCONT) ? A + r * lda + hh * KH : A + hh * KH * lda + r;
  const float* bp = (BM == KCONT) ? B + r * ldb + hh * KH : B + hh * KH * ldb + r;
#pragma unroll 4
  for (int s = 0; s < KH; s += 4) {
    float a[4], b[4];
    if (AM == KCONT) {
      const float4 t = *reinterpret_cast<const float4*>(ap + s);
      a[0] = t.x; a[1] = t.y; a[2] = t.z; a[3] = t.w;
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) a[u] = ap[(s + u) * lda];
    }
    if (BM == KCONT) {
      const float4 t = *reinterpret_cast<const float4*>(bp + s);
      b[0] = t.x; b[1] = t.y; b[2] = t.z; b[3] = t.w;
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) b[u] = bp[(s + u) * ldb];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc, 0, 0, 0);
  }
}

// The same four elements as a lane fetched them, not yet dequantised: lets a kernel
// request the rows of its next tile before the current one is multiplied and decode them
// only when they are staged.
template <int BITS>
struct RawChunk {
  static constexpr int NW = BITS == 32 ? 4 : 1;
  uint32_t w[NW];
  float z, s;
  __device__ __forceinline__ void load(const Source& src, int64_t c) {
    if (BITS == 32) {
      const float4 v = reinterpret_cast<const float4*>(src.data)[c];
      w[0] = __float_as_uint(v.x); w[1 % NW] = __float_as_uint(v.y);
      w[2 % NW] = __float_as_uint(v.z); w[3 % NW] = __float_as_uint(v.w);
      z = 0.f; s = 0.f;
      return;
    }
    if (BITS == 8) w[0] = reinterpret_cast<const uint32_t*>(src.data)[c];
    else if (BITS == 4) w[0] = reinterpret_cast<const uint16_t*>(src.data)[c];
    else if (BITS == 2) w[0] = src.data[c];
    else w[0] = (src.data[c >> 1] >> ((c & 1) * 4)) & 0xFu;
    const int64_t g = c >> src.group_chunks_log2;
    z = src.gmin[g]; s = src.gscale[g];
  }
  __device__ __forceinline__ float4 get() const {
    if (BITS == 32)
      return make_float4(__uint_as_float(w[0]), __uint_as_float(w[1 % NW]), __uint_as_float(w[2 % NW]),
                         __uint_as_float(w[3 % NW]));
    constexpr uint32_t B = (BITS == 32) ? 0u : ((1u << (BITS & 31)) - 1u);
    constexpr int SH = BITS & 31;
    float4 v;
    v.x = fmaf((float)(w[0] & B), s, z);
    v.y = fmaf((float)((w[0] >> SH) & B), s, z);
    v.z = fmaf((float)((w[0] >> (2 * SH)) & B), s, z);
    v.w = fmaf((float)((w[0] >> (3 * SH)) & B), s, z);
    return v;
  }
};

struct ChunkList {
  const int32_t* rel;
  const int32_t* start;
  const int32_t* count;
};

// ------------------------------------------------------------------ scores ----
// Half of one activation row (D/2 consecutive elements) as a lane fetched it: raw
// words plus the group's (min, scale); dequantised (Eq. 4) only when consumed, so a
// prefetched row costs D/2 * bits / 32 registers.
template <int D, int BITS>
struct HalfRow {
  static constexpr int KH = D / 2;
  static constexpr int EB = BITS == 32 ? 32 : BITS;
  static constexpr int NW = (KH * EB + 31) / 32;
  uint32_t w[NW];
  float z, s;

  __device__ __forceinline__ void load(const Source& src, int64_t node, int hh) {
    const int64_t f0 = node * D + hh * KH;   // first element; KH*EB bits, aligned to its size
    if (BITS == 32) {
      const float4* p = reinterpret_cast<const float4*>(src.data) + (f0 >> 2);
#pragma unroll
      for (int i = 0; i < KH / 4; ++i) {
        const float4 v = p[i];
        w[4 * i + 0] = __float_as_uint(v.x); w[4 * i + 1] = __float_as_uint(v.y);
        w[4 * i + 2] = __float_as_uint(v.z); w[4 * i + 3] = __float_as_uint(v.w);
      }
      z = 0.f; s = 0.f;
    } else {
      const uint8_t* p = src.data + ((f0 * EB) >> 3);
      if (KH * EB == 16) {
        w[0] = *reinterpret_cast<const uint16_t*>(p);
      } else if (NW == 1) {
        w[0] = *reinterpret_cast<const uint32_t*>(p);
      } else if (NW == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        w[0] = v.x; w[NW > 1 ? 1 : 0] = v.y;
      } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i) {
          const uint4 v = reinterpret_cast<const uint4*>(p)[i];
          w[(4 * i + 0) % NW] = v.x; w[(4 * i + 1) % NW] = v.y;
          w[(4 * i + 2) % NW] = v.z; w[(4 * i + 3) % NW] = v.w;
        }
      }
      const int64_t g = f0 >> (src.group_chunks_log2 + 2);
      z = src.gmin[g]; s = src.gscale[g];
    }
  }
  // the integer code of element i (compressed rows only)
  __device__ __forceinline__ uint32_t code(int i) const {
    constexpr uint32_t B = (1u << (EB & 31)) - 1u;
    return (w[((i * EB) >> 5) % NW] >> ((i * EB) & 31)) & B;
  }
  __device__ __forceinline__ float get(int i) const {
    if (BITS == 32) return __uint_as_float(w[i % NW]);
    constexpr uint32_t B = (1u << (EB & 31)) - 1u;
    const uint32_t code = (w[((i * EB) >> 5) % NW] >> ((i * EB) & 31)) & B;
    return fmaf((float)code, s, z);
  }
};

// ---- fp32 products on the bf16 matrix cores -------------------------------------------
// An fp32 number is the exact sum of three bfloat16 numbers (8 + 8 + 8 significant bits,
// taken by truncation): x = h + m + l.  A product x y is then h h' + (h m' + m h') +
// (m m' + h l' + l h') up to terms below 2^-23 |x y| -- the size of fp32's own rounding --
// so an fp32 contraction becomes six bf16 MFMAs (v_mfma_f32_32x32x16_bf16, fp32 accumulate),
// which run sixteen times faster than the fp32 MFMA each: 2.7 times the fp32 matrix rate at
// fp32 accuracy.  The splitting is vector work (two subtractions, two masks and 1.5 byte
// permutes per element) that overlaps with the matrix pipe.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));


union Bf16Frag {          // eight consecutive k-values of one operand row / column
  bf16x8 v;
  uint32_t u[4];
};

// Pieces of eight fp32 values: element 2i in the low half of word i, 2i + 1 in the high half.
__device__ __forceinline__ void split3x8(const float (&x)[8], Bf16Frag& h, Bf16Frag& m, Bf16Frag& l) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t hb[2], mb[2], lb[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const float v = x[2 * i + u];
      hb[u] = __float_as_uint(v) & 0xFFFF0000u;
      const float r1 = v - __uint_as_float(hb[u]);           // exact
      mb[u] = __float_as_uint(r1) & 0xFFFF0000u;
      lb[u] = __float_as_uint(r1 - __uint_as_float(mb[u]));  // exact; its upper half is kept
    }
    h.u[i] = __builtin_amdgcn_perm(hb[1], hb[0], 0x07060302u);
    m.u[i] = __builtin_amdgcn_perm(mb[1], mb[0], 0x07060302u);
    l.u[i] = __builtin_amdgcn_perm(lb[1], lb[0], 0x07060302u);
  }
}

// acc += W x for the pieces of eight k-values (six piece products, small ones first)
__device__ __forceinline__ void mfma_split(const Bf16Frag& wh, const Bf16Frag& wm, const Bf16Frag& wl,
                                           const Bf16Frag& xh, const Bf16Frag& xm, const Bf16Frag& xl,
                                           floatx16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wl.v, xh.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh.v, xl.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm.v, xm.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm.v, xh.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh.v, xm.v, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh.v, xh.v, acc, 0, 0, 0);
}

// W_r (fp32, [D][D] row-major in global memory) as three bf16 matrices in LDS, rows padded
// to D + 8 halves (row stride = 16 bytes mod 128: the 128-bit row reads of 32 lanes that
// hold 32 different rows spread over all banks).
template <int D, int LDW = D + 8>
__device__ __forceinline__ void stage_split_matrix(const float* __restrict__ W, uint16_t* __restrict__ Wp,
                                                   int tid, int n_threads) {
  constexpr int LPR = D / 4;
  for (int q = tid; q < D * LPR; q += n_threads) {
    const float4 w = reinterpret_cast<const float4*>(W)[q];
    const float x[4] = {w.x, w.y, w.z, w.w};
    uint32_t hb[4], mb[4], lb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      hb[u] = __float_as_uint(x[u]) & 0xFFFF0000u;
      const float r1 = x[u] - __uint_as_float(hb[u]);
      mb[u] = __float_as_uint(r1) & 0xFFFF0000u;
      lb[u] = __float_as_uint(r1 - __uint_as_float(mb[u]));
    }
    const int at = (q / LPR) * LDW + (q % LPR) * 4;    // in halves
    *reinterpret_cast<uint2*>(Wp + at) = make_uint2(__builtin_amdgcn_perm(hb[1], hb[0], 0x07060302u),
                                                    __builtin_amdgcn_perm(hb[3], hb[2], 0x07060302u));
    *reinterpret_cast<uint2*>(Wp + D * LDW + at) = make_uint2(__builtin_amdgcn_perm(mb[1], mb[0], 0x07060302u),
                                                              __builtin_amdgcn_perm(mb[3], mb[2], 0x07060302u));
    *reinterpret_cast<uint2*>(Wp + 2 * D * LDW + at) = make_uint2(__builtin_amdgcn_perm(lb[1], lb[0], 0x07060302u),
                                                                  __builtin_amdgcn_perm(lb[3], lb[2], 0x07060302u));
  }
}

constexpr int kScoreWaves = 4;

// Scores for d <= 64.  One wave owns 32 relation-order edges end to end: it fetches (and
// dequantises) the two rows of each edge straight into operand registers, multiplies them
// with all of W_r (split once per chunk into three bfloat16 matrices in LDS, the only shared
// state) on the bf16 matrix cores and reduces a . tanh(b) inside the wave; no workgroup
// barrier after W_r is staged.  Lane l = (r, hh)
// holds elements [32 hh, +D/2) of both rows of edge r; MFMA number m of a row block takes
// its elements [8 m, +8) -- the same permutation of the contraction index on the W_r side.
// CODES (compressed rows whose group covers at least a row, so that a row has ONE (Z, scale)
// pair): W_r e_hat = scale (W_r code) + Z (W_r 1) by Eq. (4).  The integer codes are exact
// bfloat16 values, so the product needs three piece products instead of six and no splitting or
// dequantising of the rows at all; the affine part is applied to the 32 x 32 results.
template <int D, int BITS, bool CODES>
__global__ __launch_bounds__(kScoreWaves * 64) void score_split_kernel(Source src, const float* __restrict__ Wr,
                                                               const float* __restrict__ er,
                                                               const int32_t* __restrict__ r_head,
                                                               const int32_t* __restrict__ r_tail,
                                                               const int32_t* __restrict__ r_eid,
                                                               ChunkList chunks, float* __restrict__ s_out) {
  constexpr int LDW = D + 8, KH = D / 2, NCB = D / 32, NM = KH / 8;
  static_assert(!CODES || BITS != 32, "codes exist for compressed rows only");
  uint16_t* Wp = reinterpret_cast<uint16_t*>(smem_raw);                 // [3][D][LDW] halves
  float* er_s = reinterpret_cast<float*>(Wp + 3 * D * LDW);
  float* wsum_s = er_s + D;                                             // row sums of W_r (CODES)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ch = blockIdx.x;
  const int rel = chunks.rel[ch], start = chunks.start[ch], count = chunks.count[ch];
  const int r = lane & 31, hh = lane >> 5;
  const int n_wt = (count + 31) >> 5;
  int wt = wave;

  int t_nx = 0, h_nx = 0, e_nx = -1;
  auto load_idx = [&](int tile) {
    const int row = tile * 32 + r;
    t_nx = 0; h_nx = 0; e_nx = -1;
    if (row < count) { const int pos = start + row; t_nx = r_tail[pos]; h_nx = r_head[pos]; e_nx = r_eid[pos]; }
  };
  HalfRow<D, BITS> nt, nh;

  stage_split_matrix<D>(Wr + (size_t)rel * D * D, Wp, tid, kScoreWaves * 64);
  for (int c = tid; c < D; c += kScoreWaves * 64) er_s[c] = er[(size_t)rel * D + c];
  if (CODES) {
    for (int c = tid; c < D; c += kScoreWaves * 64) {
      const float4* row = reinterpret_cast<const float4*>(Wr + ((size_t)rel * D + c) * D);
      double sum = 0.0;
      for (int q = 0; q < D / 4; ++q) { const float4 w = row[q]; sum += (double)w.x + (double)w.y + (double)w.z + (double)w.w; }
      wsum_s[c] = (float)sum;
    }
  }
  __syncthreads();
  if (wt >= n_wt) return;

  for (; wt < n_wt; wt += kScoreWaves) {
    // (rows fetched here, not a tile ahead: the raw words of a prefetched tile cost a wave per
    // SIMD in registers, and the other waves cover the latency better than the prefetch did)
    load_idx(wt);
    nt.load(src, t_nx, hh);
    nh.load(src, h_nx, hh);
    float tv[CODES ? 1 : KH], hv[CODES ? 1 : KH];
    Bf16Frag tc[CODES ? NM : 1], hc[CODES ? NM : 1];
    float zt = 0.f, st = 0.f, zh = 0.f, sh = 0.f;
    if constexpr (CODES) {
      auto pack = [](uint32_t c0, uint32_t c1) {     // two codes as bfloat16 values (exact)
        return __builtin_amdgcn_perm(__float_as_uint((float)c1), __float_as_uint((float)c0), 0x07060302u);
      };
#pragma unroll
      for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          tc[m].u[i] = pack(nt.code(8 * m + 2 * i), nt.code(8 * m + 2 * i + 1));
          hc[m].u[i] = pack(nh.code(8 * m + 2 * i), nh.code(8 * m + 2 * i + 1));
        }
      zt = nt.z; st = nt.s; zh = nh.z; sh = nh.s;
    } else {
#pragma unroll
      for (int i = 0; i < KH; ++i) { tv[i] = nt.get(i); hv[i] = nh.get(i); }
    }
    const int eid = e_nx;
    floatx16 accA[NCB], accB[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      accA[cb] = floatx16{0};
#pragma unroll
      for (int v = 0; v < 16; ++v) accB[cb][v] = CODES ? 0.f : er_s[cb * 32 + acc_row(v, lane)];
    }
    int wofs = 0;
    asm volatile("" : "+v"(wofs));
    const uint16_t* wrow = Wp + r * LDW + hh * KH + wofs;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      Bf16Frag th, tm, tl, hhi, hmi, hlo;
      if constexpr (!CODES) {
        float a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { a[i] = tv[8 * m + i]; b[i] = hv[8 * m + i]; }
        split3x8(a, th, tm, tl);
        split3x8(b, hhi, hmi, hlo);
      }
      Bf16Frag wh[NCB], wm[NCB], wl[NCB];
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const uint16_t* wp = wrow + cb * 32 * LDW + 8 * m;
        *reinterpret_cast<uint4*>(wh[cb].u) = *reinterpret_cast<const uint4*>(wp);
        *reinterpret_cast<uint4*>(wm[cb].u) = *reinterpret_cast<const uint4*>(wp + D * LDW);
        *reinterpret_cast<uint4*>(wl[cb].u) = *reinterpret_cast<const uint4*>(wp + 2 * D * LDW);
      }
      // six piece products (small ones first), each over the 2 NCB independent accumulators
#define TINYKG_SPLIT_STEP(WP, TP, HP)                                                                      \
      _Pragma("unroll") for (int cb = 0; cb < NCB; ++cb) {                                                 \
        accA[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WP[cb].v, TP.v, accA[cb], 0, 0, 0);             \
        accB[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WP[cb].v, HP.v, accB[cb], 0, 0, 0);             \
      }
      if constexpr (CODES) {
        TINYKG_SPLIT_STEP(wl, tc[m], hc[m])
        TINYKG_SPLIT_STEP(wm, tc[m], hc[m])
        TINYKG_SPLIT_STEP(wh, tc[m], hc[m])
      } else {
        TINYKG_SPLIT_STEP(wl, th, hhi)
        TINYKG_SPLIT_STEP(wh, tl, hlo)
        TINYKG_SPLIT_STEP(wm, tm, hmi)
        TINYKG_SPLIT_STEP(wm, th, hhi)
        TINYKG_SPLIT_STEP(wh, tm, hmi)
        TINYKG_SPLIT_STEP(wh, th, hhi)
      }
#undef TINYKG_SPLIT_STEP
    }
    float p = 0.f;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if constexpr (CODES) {
          const int c = cb * 32 + acc_row(v, lane);
          const float ws = wsum_s[c];
          const float a = fmaf(st, accA[cb][v], zt * ws);
          const float b = fmaf(sh, accB[cb][v], fmaf(zh, ws, er_s[c]));
          p = fmaf(a, fast_tanh(b), p);
        } else {
          p = fmaf(accA[cb][v], fast_tanh(accB[cb][v]), p);
        }
      }
    }
    p += __shfl_xor(p, 32);
    if (hh == 0 && eid >= 0) s_out[eid] = p;
  }
}

// Three bf16 pieces of four consecutive fp32 values, stored at the same position of three
// LDS matrices `piece_stride` halves apart.
__device__ __forceinline__ void store_split4(const float4& v, uint16_t* dst, int piece_stride) {
  const float x[4] = {v.x, v.y, v.z, v.w};
  uint32_t hb[4], mb[4], lb[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    hb[u] = __float_as_uint(x[u]) & 0xFFFF0000u;
    const float r1 = x[u] - __uint_as_float(hb[u]);
    mb[u] = __float_as_uint(r1) & 0xFFFF0000u;
    lb[u] = __float_as_uint(r1 - __uint_as_float(mb[u]));
  }
  *reinterpret_cast<uint2*>(dst) = make_uint2(__builtin_amdgcn_perm(hb[1], hb[0], 0x07060302u),
                                              __builtin_amdgcn_perm(hb[3], hb[2], 0x07060302u));
  *reinterpret_cast<uint2*>(dst + piece_stride) = make_uint2(__builtin_amdgcn_perm(mb[1], mb[0], 0x07060302u),
                                                             __builtin_amdgcn_perm(mb[3], mb[2], 0x07060302u));
  *reinterpret_cast<uint2*>(dst + 2 * piece_stride) = make_uint2(__builtin_amdgcn_perm(lb[1], lb[0], 0x07060302u),
                                                                 __builtin_amdgcn_perm(lb[3], lb[2], 0x07060302u));
}

// The four integer codes of a compressed chunk as bfloat16 values (exact), to LDS.
template <int BITS>
__device__ __forceinline__ void store_codes4(const RawChunk<BITS>& c, uint16_t* dst) {
  constexpr uint32_t B = (BITS == 32) ? 0u : ((1u << (BITS & 31)) - 1u);
  constexpr int SH = BITS & 31;
  const uint32_t w = c.w[0];
  const uint32_t f0 = __float_as_uint((float)(w & B)), f1 = __float_as_uint((float)((w >> SH) & B));
  const uint32_t f2 = __float_as_uint((float)((w >> (2 * SH)) & B)), f3 = __float_as_uint((float)((w >> (3 * SH)) & B));
  *reinterpret_cast<uint2*>(dst) = make_uint2(__builtin_amdgcn_perm(f1, f0, 0x07060302u),
                                              __builtin_amdgcn_perm(f3, f2, 0x07060302u));
}

// Scores for d = 128, cooperative 32-edge tiles.  Wave w of the four owns channel block w
// for the whole chunk and keeps its 32 x 128 block of W_r, split into the three bfloat16
// pieces, in REGISTERS (96 per lane: one wave per SIMD and workgroup, so the registers are
// there, and LDS -- which three pieces of the whole W_r would fill to two thirds -- holds only
// the tile).  That leaves room for two workgroups per compute unit, whose barrier-separated
// phases (stage the tile / multiply) overlap each other.  The tile's rows are split as they
// are staged (once per element, whatever the number of waves that multiply them); a wave then
// reads ready 128-bit fragments.  k-step m of half hh covers k = 16 m + 8 hh + 0..7 on both
// operands.
// (CODES: as in score_split_kernel -- the tile holds one bfloat16 matrix of codes per side and
// the rows' (Z, scale) pairs instead of three pieces of dequantised values)
template <int D, int TE, int BITS, bool CODES>
__global__ __launch_bounds__(kThreads, 2) void score_coop_split_kernel(Source src, const float* __restrict__ Wr,
                                                                       const float* __restrict__ er,
                                                                       const int32_t* __restrict__ r_head,
                                                                       const int32_t* __restrict__ r_tail,
                                                                       const int32_t* __restrict__ r_eid,
                                                                       ChunkList chunks, float* __restrict__ s_out) {
  constexpr int LDW = D + 8, LPR = D / 4, NCB = D / 32, NP = NCB * 2, NM = D / 16;
  constexpr int CPT = TE * LPR / kThreads, RSTEP = kThreads / LPR;
  constexpr int TP = TE * LDW;                    // halves per piece
  constexpr int NPIECE = CODES ? 1 : 3;
  static_assert(TE == 32 && NCB * 64 == kThreads, "one 32 x 32 block of a and of b per wave and tile");
  static_assert(TE * LPR % kThreads == 0 && kThreads % LPR == 0, "tile does not split evenly");
  uint16_t* Et_s = reinterpret_cast<uint16_t*>(smem_raw);        // [NPIECE][TE][LDW]
  uint16_t* Eh_s = Et_s + NPIECE * TP;
  float* er_s = reinterpret_cast<float*>(Eh_s + NPIECE * TP);
  float* part = er_s + D;  // [NP][TE]
  float* wsum_s = part + NP * TE;      // [D] row sums of W_r           (CODES)
  float* zs_s = wsum_s + D;            // [4][TE] Z_t, scale_t, Z_h, scale_h of the tile's rows (CODES)
  static_assert(!CODES || BITS != 32, "codes exist for compressed rows only");

  const int tid = threadIdx.x, lane = tid & 63, cb = tid >> 6;
  const int ch = blockIdx.x;
  const int r = chunks.rel[ch], start = chunks.start[ch], count = chunks.count[ch];
  const int row0 = tid / LPR, li = tid % LPR;

  int tn[CPT], hn[CPT];
  auto load_ids = [&](int t0) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int row = t0 + row0 + k * RSTEP;
      tn[k] = 0; hn[k] = 0;
      if (row < count) { tn[k] = r_tail[start + row]; hn[k] = r_head[start + row]; }
    }
  };
  RawChunk<BITS> rt[CPT], rh[CPT];
  auto load_rows = [&]() {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      rt[k].load(src, (int64_t)tn[k] * LPR + li);
      rh[k].load(src, (int64_t)hn[k] * LPR + li);
    }
  };
  load_ids(0);
  load_rows();
  load_ids(TE);

  // this wave's block of W_r: row cb * 32 + (lane & 31), k-values 16 m + 8 (lane >> 5) + 0..7
  Bf16Frag wh[NM], wm[NM], wl[NM];
  {
    const float* wrow = Wr + ((size_t)r * D + cb * 32 + (lane & 31)) * D + (lane >> 5) * 8;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const float4 lo4 = *reinterpret_cast<const float4*>(wrow + 16 * m);
      const float4 hi4 = *reinterpret_cast<const float4*>(wrow + 16 * m + 4);
      const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
      split3x8(x, wh[m], wm[m], wl[m]);
    }
  }
  for (int c = tid; c < D; c += kThreads) er_s[c] = er[(size_t)r * D + c];
  if (CODES) {
    for (int c = tid; c < D; c += kThreads) {
      const float4* row = reinterpret_cast<const float4*>(Wr + ((size_t)r * D + c) * D);
      double sum = 0.0;
      for (int q = 0; q < D / 4; ++q) { const float4 w = row[q]; sum += (double)w.x + (double)w.y + (double)w.z + (double)w.w; }
      wsum_s[c] = (float)sum;
    }
  }

  for (int t0 = 0; t0 < count; t0 += TE) {
    const int nrow = min(TE, count - t0);
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int row = row0 + k * RSTEP;
      if constexpr (CODES) {
        store_codes4(rt[k], Et_s + row * LDW + li * 4);
        store_codes4(rh[k], Eh_s + row * LDW + li * 4);
        if (li == 0) {
          zs_s[row] = rt[k].z; zs_s[TE + row] = rt[k].s;
          zs_s[2 * TE + row] = rh[k].z; zs_s[3 * TE + row] = rh[k].s;
        }
      } else {
        store_split4(rt[k].get(), Et_s + row * LDW + li * 4, TP);
        store_split4(rh[k].get(), Eh_s + row * LDW + li * 4, TP);
      }
    }
    if (t0 + TE < count) {
      load_rows();
      load_ids(t0 + 2 * TE);
    }
    __syncthreads();
    {
      floatx16 accA = {0}, accB = {0};
      const int fr = (lane & 31) * LDW + (lane >> 5) * 8;
      const uint16_t* tp = Et_s + fr;
      const uint16_t* hp = Eh_s + fr;
      auto ld = [](const uint16_t* p) { Bf16Frag f; *reinterpret_cast<uint4*>(f.u) = *reinterpret_cast<const uint4*>(p); return f; };
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const Bf16Frag th = ld(tp + 16 * m), hh_ = ld(hp + 16 * m);
#define TINYKG_SPLIT_STEP(WF, TF, HF)                                                           \
        accA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WF[m].v, TF.v, accA, 0, 0, 0);           \
        accB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WF[m].v, HF.v, accB, 0, 0, 0);
        if constexpr (CODES) {
          TINYKG_SPLIT_STEP(wl, th, hh_)
          TINYKG_SPLIT_STEP(wm, th, hh_)
          TINYKG_SPLIT_STEP(wh, th, hh_)
        } else {
          const Bf16Frag tm = ld(tp + TP + 16 * m), tl = ld(tp + 2 * TP + 16 * m);
          const Bf16Frag hm = ld(hp + TP + 16 * m), hl = ld(hp + 2 * TP + 16 * m);
          TINYKG_SPLIT_STEP(wl, th, hh_)
          TINYKG_SPLIT_STEP(wh, tl, hl)
          TINYKG_SPLIT_STEP(wm, tm, hm)
          TINYKG_SPLIT_STEP(wm, th, hh_)
          TINYKG_SPLIT_STEP(wh, tm, hm)
          TINYKG_SPLIT_STEP(wh, th, hh_)
        }
#undef TINYKG_SPLIT_STEP
      }
      float p = 0.f;
      float zt = 0.f, st = 0.f, zh = 0.f, sh = 0.f;
      if constexpr (CODES) {
        const int e = lane & 31;
        zt = zs_s[e]; st = zs_s[TE + e]; zh = zs_s[2 * TE + e]; sh = zs_s[3 * TE + e];
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int c = cb * 32 + acc_row(v, lane);
        if constexpr (CODES) {
          const float ws = wsum_s[c];
          const float a = fmaf(st, accA[v], zt * ws);
          p = fmaf(a, fast_tanh(fmaf(sh, accB[v], fmaf(zh, ws, er_s[c]))), p);
        } else {
          p = fmaf(accA[v], fast_tanh(accB[v] + er_s[c]), p);
        }
      }
      part[(cb * 2 + (lane >> 5)) * TE + (lane & 31)] = p;
    }
    __syncthreads();
    if (tid < nrow) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < NP; ++k) s += part[k * TE + tid];
      s_out[r_eid[start + t0 + tid]] = s;
    }
  }
}

// ---------------------------------------------------------- per-head stages ----
// Sum over the LPR (8, 16 or 32) adjacent lanes that share one edge, result on every one
// of them: DPP steps inside a row of 16 lanes (after each step the reduced sub-block is
// uniform, so a mirror pairs it with its neighbour), one cross-lane exchange for 32.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int LPR>
__device__ __forceinline__ float slot_sum(float v) {
  v += dpp_f<0xB1>(v);                    // quad_perm:[1,0,3,2]
  v += dpp_f<0x4E>(v);                    // quad_perm:[2,3,0,1]
  if (LPR >= 8) v += dpp_f<0x141>(v);     // row_half_mirror
  if (LPR >= 16) v += dpp_f<0x140>(v);    // row_mirror
  if (LPR >= 32) v += __shfl_xor(v, 16);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <int LPR>
__device__ __forceinline__ float slot_max(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  if (LPR >= 8) v = fmaxf(v, dpp_f<0x141>(v));
  if (LPR >= 16) v = fmaxf(v, dpp_f<0x140>(v));
  if (LPR >= 32) v = fmaxf(v, __shfl_xor(v, 16));
  return v;
}

// Softmax statistics of the scores of one head's out-edges [e0, e0+deg), by a whole wave.
// At most kHeavyDegree terms (longer neighbourhoods take the segment kernels, which sum in
// double): fp32 sums.
__device__ __forceinline__ void softmax_stats(const float* __restrict__ s, int e0, int deg, int lane,
                                              float& m, float& z) {
  m = -INFINITY;
  for (int i = lane; i < deg; i += 64) m = fmaxf(m, s[e0 + i]);
  m = wave_max(m);
  float zs = 0.f;
  for (int i = lane; i < deg; i += 64) zs += __expf(s[e0 + i] - m);
  z = wave_sum(zs);
}

// Softmax weights of a short neighbourhood (at most kSlotDegree edges) owned by a slot of LPR
// lanes: lane li computes the weights of edges li, li + LPR, ... ONCE (one exponential per edge
// and one reciprocal per lane instead of one of each per edge and lane); slot_weight hands
// edge j's weight to every lane of the slot.  exp through the hardware exp2 unit: relative
// error about 1e-7 (1 + |x|) on a weight exp(x), x <= 0.
constexpr int kSlotDegree = 16;
template <int LPR>
constexpr int kSlotWeights = (kSlotDegree + LPR - 1) / LPR;

template <int LPR>
__device__ __forceinline__ void slot_softmax(const float* __restrict__ s, int e0, int ds, int li,
                                             float (&pw)[kSlotWeights<LPR>]) {
  float sc[kSlotWeights<LPR>];
  float m = -INFINITY;
#pragma unroll
  for (int q = 0; q < kSlotWeights<LPR>; ++q) {
    const int j = li + q * LPR;
    sc[q] = j < ds ? s[e0 + j] : -INFINITY;
    m = fmaxf(m, sc[q]);
  }
  m = slot_max<LPR>(m);
  if (ds == 0) m = 0.f;
  float z = 0.f;
#pragma unroll
  for (int q = 0; q < kSlotWeights<LPR>; ++q) { pw[q] = __expf(sc[q] - m); z += pw[q]; }   // exp(-inf) = 0
  z = slot_sum<LPR>(z);
  const float inv = ds == 0 ? 0.f : 1.0f / z;
#pragma unroll
  for (int q = 0; q < kSlotWeights<LPR>; ++q) pw[q] *= inv;
}

template <int LPR>
__device__ __forceinline__ float slot_weight(const float (&pw)[kSlotWeights<LPR>], int j, int lane) {
  return __shfl(pw[j / LPR], (lane & ~(LPR - 1)) | (j % LPR));
}

// The per-head kernels take 64 / LPR consecutive heads per wave and step (LPR = D / 4 lanes
// hold one row).  A head with at most kSlotDegree out-edges is handled by ONE slot of LPR
// lanes, so several short neighbourhoods -- the common case: the mean out-degree of a
// knowledge graph is around ten -- advance side by side and pay the per-head latencies
// (row pointers, statistics, dependent gathers) together.  Heads between kSlotDegree and
// kHeavyDegree are then taken one at a time by the whole wave, 64 / LPR edges per step.

template <int D, int BITS>
__global__ __launch_bounds__(kThreads) void attend_fwd_kernel(Source src,
                                                              const int32_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ h_tail,
                                                              const float* __restrict__ s, int64_t N,
                                                              float* __restrict__ H) {
  constexpr int LPR = D / 4, ES = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int sub = lane / LPR, li = lane % LPR;
  const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
  for (int64_t h0 = ((int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)) * ES; h0 < N;
       h0 += n_waves * ES) {
    const int64_t h = h0 + sub;
    int e0 = 0, deg = 0;
    if (h < N) { e0 = rowptr[h]; deg = rowptr[h + 1] - e0; }
    const bool small = deg <= kSlotDegree;
    // ---- short neighbourhoods: one slot per head
    {
      const int ds = small ? deg : 0;
      float pw[kSlotWeights<LPR>];
      slot_softmax<LPR>(s, e0, ds, li, pw);
      float ax = 0.f, ay = 0.f, az = 0.f, aw = 0.f;
#pragma unroll
      for (int j0 = 0; j0 < kSlotDegree; j0 += 4) {
        if (__builtin_amdgcn_ballot_w64(j0 < ds) == 0) break;
        int t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = j0 + u < ds ? h_tail[e0 + j0 + u] : 0;   // unused places: node 0, weight 0
        float4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = fetch_chunk<BITS>(src, (int64_t)t[u] * LPR + li);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float p = slot_weight<LPR>(pw, j0 + u, lane);
          ax = fmaf(p, x[u].x, ax); ay = fmaf(p, x[u].y, ay);
          az = fmaf(p, x[u].z, az); aw = fmaf(p, x[u].w, aw);
        }
      }
      if (h < N && small) {
        const float4 eh = fetch_chunk<BITS>(src, h * LPR + li);
        reinterpret_cast<float4*>(H)[h * LPR + li] = make_float4(eh.x + ax, eh.y + ay, eh.z + az, eh.w + aw);
      }
    }
    // ---- longer ones: the whole wave, one head at a time (heavy heads: the heavy_* kernels)
    uint64_t pend = __builtin_amdgcn_ballot_w64(!small && deg <= kHeavyDegree && li == 0);
    while (pend) {
      const int leader = __builtin_amdgcn_readfirstlane(__ffsll((long long)pend) - 1);
      pend &= pend - 1;
      const int64_t hw = h0 + leader / LPR;
      const int e0w = __builtin_amdgcn_readlane(e0, leader), degw = __builtin_amdgcn_readlane(deg, leader);
      float m, z;
      softmax_stats(s, e0w, degw, lane, m, z);
      float ax = 0.f, ay = 0.f, az = 0.f, aw = 0.f;
      for (int base = 0; base < degw; base += ES) {
        const int j = base + sub;
        if (j < degw) {
          const float p = __expf(s[e0w + j] - m) * (1.0f / z);
          const float4 x = fetch_chunk<BITS>(src, (int64_t)h_tail[e0w + j] * LPR + li);
          ax = fmaf(p, x.x, ax); ay = fmaf(p, x.y, ay);
          az = fmaf(p, x.z, az); aw = fmaf(p, x.w, aw);
        }
      }
#pragma unroll
      for (int o = LPR; o < 64; o <<= 1) {
        ax += __shfl_xor(ax, o); ay += __shfl_xor(ay, o);
        az += __shfl_xor(az, o); aw += __shfl_xor(aw, o);
      }
      if (sub == 0) {
        const float4 eh = fetch_chunk<BITS>(src, hw * LPR + li);
        reinterpret_cast<float4*>(H)[hw * LPR + li] = make_float4(eh.x + ax, eh.y + ay, eh.z + az, eh.w + aw);
      }
    }
  }
}

template <int D, int BITS>
__global__ __launch_bounds__(kThreads) void attend_bwd_kernel(Source src, const float* __restrict__ gH,
                                                              const int32_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ h_tail,
                                                              const float* __restrict__ s, int64_t N,
                                                              float* __restrict__ pi,
                                                              float* __restrict__ gs) {
  constexpr int LPR = D / 4, ES = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int sub = lane / LPR, li = lane % LPR;
  const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
  const float4* G4 = reinterpret_cast<const float4*>(gH);
  for (int64_t h0 = ((int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)) * ES; h0 < N;
       h0 += n_waves * ES) {
    const int64_t h = h0 + sub;
    int e0 = 0, deg = 0;
    if (h < N) { e0 = rowptr[h]; deg = rowptr[h + 1] - e0; }
    const bool small = deg <= kSlotDegree;
    // ---- short neighbourhoods: one slot per head; pi_j, g_j stay in registers until
    //      c = sum pi_j g_j is known, so grad_s_j = pi_j (g_j - c) is written once
    {
      const int ds = small ? deg : 0;
      float pw[kSlotWeights<LPR>];
      slot_softmax<LPR>(s, e0, ds, li, pw);
      float4 g4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (ds > 0) g4 = G4[h * LPR + li];
      float pj[kSlotDegree], gj[kSlotDegree];
      float c = 0.f;
#pragma unroll
      for (int j0 = 0; j0 < kSlotDegree; j0 += 4) {
        const bool any = __builtin_amdgcn_ballot_w64(j0 < ds) != 0;    // wave-uniform
        int t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = (any && j0 + u < ds) ? h_tail[e0 + j0 + u] : 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          float dot = 0.f;
          if (any) {
            const float4 x = fetch_chunk<BITS>(src, (int64_t)t[u] * LPR + li);
            dot = fmaf(g4.x, x.x, fmaf(g4.y, x.y, fmaf(g4.z, x.z, g4.w * x.w)));
            dot = slot_sum<LPR>(dot);
          }
          const float p = slot_weight<LPR>(pw, j0 + u, lane);     // 0 for unused places
          pj[j0 + u] = p;
          gj[j0 + u] = dot;
          c = fmaf(p, dot, c);
        }
      }
      if (li == 0) {
#pragma unroll
        for (int j = 0; j < kSlotDegree; ++j)
          if (j < ds) { pi[e0 + j] = pj[j]; gs[e0 + j] = pj[j] * (gj[j] - c); }
      }
    }
    // ---- longer ones: the whole wave, one head at a time (heavy heads: the heavy_* kernels)
    uint64_t pend = __builtin_amdgcn_ballot_w64(!small && deg <= kHeavyDegree && li == 0);
    while (pend) {
      const int leader = __builtin_amdgcn_readfirstlane(__ffsll((long long)pend) - 1);
      pend &= pend - 1;
      const int64_t hw = h0 + leader / LPR;
      const int e0w = __builtin_amdgcn_readlane(e0, leader), degw = __builtin_amdgcn_readlane(deg, leader);
      float m, z;
      softmax_stats(s, e0w, degw, lane, m, z);
      const float4 g4 = G4[hw * LPR + li];
      float cpart = 0.f;
      for (int base = 0; base < degw; base += ES) {
        const int j = base + sub;
        float dot = 0.f, p = 0.f;
        if (j < degw) {
          p = __expf(s[e0w + j] - m) * (1.0f / z);
          const float4 x = fetch_chunk<BITS>(src, (int64_t)h_tail[e0w + j] * LPR + li);
          dot = fmaf(g4.x, x.x, fmaf(g4.y, x.y, fmaf(g4.z, x.z, g4.w * x.w)));
        }
        dot = slot_sum<LPR>(dot);   // g_j on every lane of the slot
        if (j < degw) {
          cpart = fmaf(p, dot, cpart);
          if (li == 0) { pi[e0w + j] = p; gs[e0w + j] = dot; }
        }
      }
      float c = cpart;     // equal on the lanes of a slot: sum once per slot
#pragma unroll
      for (int o = LPR; o < 64; o <<= 1) c += __shfl_xor(c, o);
      // grad_s_j = pi_j (g_j - sum_j' pi_j' g_j'); each lane re-reads what it wrote itself
      for (int base = 0; base < degw; base += ES) {
        const int j = base + sub;
        if (j < degw && li == 0) gs[e0w + j] = pi[e0w + j] * (gs[e0w + j] - c);
      }
    }
  }
}


// ---------------------------------------------------------------- heavy heads ----
// A head with more than kHeavyDegree out-edges is processed in segments of that many
// edges, one wave per segment, and a small per-head pass merges the segments.  The
// softmax is merged in the usual shifted form: a segment keeps (m_s, z_s, acc_s) with
// z_s = sum exp(s_j - m_s), acc_s = sum exp(s_j - m_s) e_t, and the head's values are
// M = max m_s, Z = sum z_s exp(m_s - M), acc = sum acc_s exp(m_s - M).
struct HeavyList {
  const int32_t* head;     // [n_heavy]
  const int32_t* seg_ptr;  // [n_heavy + 1]
  const int32_t* seg_q;    // [n_hseg]
  const int32_t* seg_e0;   // [n_hseg]
  const int32_t* seg_cnt;  // [n_hseg]
  int n_heavy, n_hseg;
};

// Per segment: pm, pz and (WITH_ACC) the unnormalised weighted row sum pacc [n_hseg, D].
template <int D, bool WITH_ACC, int BITS>
__global__ __launch_bounds__(kThreads) void heavy_part1_kernel(Source src,
                                                               const int32_t* __restrict__ h_tail,
                                                               const float* __restrict__ s, HeavyList hl,
                                                               float* __restrict__ pm, double* __restrict__ pz,
                                                               double* __restrict__ pacc) {
  constexpr int LPR = D / 4, ES = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane / LPR, li = lane % LPR;
  const int sg = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (sg >= hl.n_hseg) return;
  const int e0 = hl.seg_e0[sg], cnt = hl.seg_cnt[sg];
  float m = -INFINITY;
  for (int i = lane; i < cnt; i += 64) m = fmaxf(m, s[e0 + i]);
  m = wave_max(m);
  double zd = 0.0;
  for (int i = lane; i < cnt; i += 64) zd += (double)expf(s[e0 + i] - m);
  zd = wave_sum(zd);
  if (lane == 0) { pm[sg] = m; pz[sg] = zd; }
  if (WITH_ACC) {
    double ax = 0.0, ay = 0.0, az = 0.0, aw = 0.0;
    for (int base = 0; base < cnt; base += ES) {
      const int j = base + sub;
      if (j < cnt) {
        const double p = (double)expf(s[e0 + j] - m);
        const float4 x = fetch_chunk<BITS>(src, (int64_t)h_tail[e0 + j] * LPR + li);
        ax = fma(p, (double)x.x, ax); ay = fma(p, (double)x.y, ay);
        az = fma(p, (double)x.z, az); aw = fma(p, (double)x.w, aw);
      }
    }
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      ax += __shfl_xor(ax, o); ay += __shfl_xor(ay, o);
      az += __shfl_xor(az, o); aw += __shfl_xor(aw, o);
    }
    if (sub == 0) {
      double* out = pacc + (int64_t)sg * D + li * 4;
      out[0] = ax; out[1] = ay; out[2] = az; out[3] = aw;
    }
  }
}

// Per heavy head (one workgroup of kMergeWaves waves): M, Z (-> hm, hz) and, WITH_ACC,
// H_h = e_h + acc / Z.  Wave w sums the segments a + w, a + w + kMergeWaves, ... in double;
// the waves' sums are then added in the order 0, 1, ... (fixed, so H is reproducible).
constexpr int kMergeWaves = 16;

template <int D, bool WITH_ACC, int BITS>
__global__ __launch_bounds__(kMergeWaves * 64) void heavy_merge1_kernel(
    Source src, HeavyList hl, const float* __restrict__ pm,
    const double* __restrict__ pz, const double* __restrict__ pacc, float* __restrict__ hm,
    double* __restrict__ hz, float* __restrict__ H) {
  __shared__ double part[kMergeWaves][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = blockIdx.x;
  const int a = hl.seg_ptr[q], b = hl.seg_ptr[q + 1];
  float M = -INFINITY;
  for (int i = a + lane; i < b; i += 64) M = fmaxf(M, pm[i]);
  M = wave_max(M);
  double Z = 0.0;
  for (int i = a + lane; i < b; i += 64) Z += pz[i] * (double)expf(pm[i] - M);
  Z = wave_sum(Z);
  if (threadIdx.x == 0) { hm[q] = M; hz[q] = Z; }
  if (WITH_ACC) {
    for (int i = lane; i < D; i += 64) {
      double acc = 0.0;
      int sgi = a + wave;
      for (; sgi + 3 * kMergeWaves < b; sgi += 4 * kMergeWaves) {      // four loads in flight
        const double p0 = pacc[(int64_t)sgi * D + i], p1 = pacc[(int64_t)(sgi + kMergeWaves) * D + i];
        const double p2 = pacc[(int64_t)(sgi + 2 * kMergeWaves) * D + i];
        const double p3 = pacc[(int64_t)(sgi + 3 * kMergeWaves) * D + i];
        const float m0 = pm[sgi], m1 = pm[sgi + kMergeWaves], m2 = pm[sgi + 2 * kMergeWaves];
        const float m3 = pm[sgi + 3 * kMergeWaves];
        acc += p0 * (double)expf(m0 - M);
        acc += p1 * (double)expf(m1 - M);
        acc += p2 * (double)expf(m2 - M);
        acc += p3 * (double)expf(m3 - M);
      }
      for (; sgi < b; sgi += kMergeWaves) acc += pacc[(int64_t)sgi * D + i] * (double)expf(pm[sgi] - M);
      part[wave][i] = acc;
    }
    __syncthreads();
    if (wave == 0) {
      const int64_t h = hl.head[q];
      for (int i = lane; i < D; i += 64) {
        double acc = 0.0;
#pragma unroll
        for (int w = 0; w < kMergeWaves; ++w) acc += part[w][i];
        const float4 e4 = fetch_chunk<BITS>(src, (h * D + i) >> 2);     // the chunk that holds column i
        const float eh = (i & 3) == 0 ? e4.x : (i & 3) == 1 ? e4.y : (i & 3) == 2 ? e4.z : e4.w;
        H[h * D + i] = (float)((double)eh + acc / Z);
      }
    }
  }
}

// Backward, per segment: pi_j = exp(s_j - M) / Z, g_j = grad_H_h . e_hat_t (kept in gs),
// and the segment's part of c = sum pi_j g_j.
template <int D, int BITS>
__global__ __launch_bounds__(kThreads) void heavy_part2_kernel(Source src, const float* __restrict__ gH,
                                                               const int32_t* __restrict__ h_tail,
                                                               const float* __restrict__ s, HeavyList hl,
                                                               const float* __restrict__ hm,
                                                               const double* __restrict__ hz,
                                                               float* __restrict__ pi, float* __restrict__ gs,
                                                               double* __restrict__ pc) {
  constexpr int LPR = D / 4, ES = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane / LPR, li = lane % LPR;
  const int sg = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (sg >= hl.n_hseg) return;
  const int e0 = hl.seg_e0[sg], cnt = hl.seg_cnt[sg], q = hl.seg_q[sg];
  const int64_t h = hl.head[q];
  const float M = hm[q];
  const float Zf = (float)hz[q];
  const float4 g4 = reinterpret_cast<const float4*>(gH)[h * LPR + li];
  double cpart = 0.0;
  for (int base = 0; base < cnt; base += ES) {
    const int j = base + sub;
    float dot = 0.f, p = 0.f;
    if (j < cnt) {
      p = expf(s[e0 + j] - M) / Zf;
      const float4 x = fetch_chunk<BITS>(src, (int64_t)h_tail[e0 + j] * LPR + li);
      dot = fmaf(g4.x, x.x, fmaf(g4.y, x.y, fmaf(g4.z, x.z, g4.w * x.w)));
    }
    dot = slot_sum<LPR>(dot);
    if (j < cnt) {
      cpart = fma((double)p, (double)dot, cpart);
      if (li == 0) { pi[e0 + j] = p; gs[e0 + j] = dot; }
    }
  }
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) cpart += __shfl_xor(cpart, o);
  if (lane == 0) pc[sg] = cpart;
}

// Backward, per segment: c = sum of the head's segment parts (fixed order), then
// grad_s_j = pi_j (g_j - c).
__global__ __launch_bounds__(kThreads) void heavy_part3_kernel(HeavyList hl, const double* __restrict__ pc,
                                                               const float* __restrict__ pi,
                                                               float* __restrict__ gs) {
  const int lane = threadIdx.x & 63;
  const int sg = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (sg >= hl.n_hseg) return;
  const int q = hl.seg_q[sg];
  const int a = hl.seg_ptr[q], b = hl.seg_ptr[q + 1];
  double c = 0.0;
  for (int i = a + lane; i < b; i += 64) c += pc[i];
  c = wave_sum(c);
  const float cf = (float)c;
  const int e0 = hl.seg_e0[sg], cnt = hl.seg_cnt[sg];
  for (int i = lane; i < cnt; i += 64) gs[e0 + i] = pi[e0 + i] * (gs[e0 + i] - cf);
}

// ------------------------------------------------------------- dense stage ----
// J = H W^T, E' = LeakyReLU(J), mask = [J > 0].  64 nodes per tile.
// A wave keeps its 32 x D block of W in registers for the whole launch, split into its three
// bfloat16 pieces (wave w: output block w mod NOB; the waves that share a block share the tile's
// two node blocks), so LDS holds only the tile and several workgroups fit a compute unit: the
// loads, the products and the stores of different workgroups overlap, which a single resident
// workgroup's barriers rule out.  The rows of H are split as they are read: six piece products
// on the bf16 matrix cores per sixteen k-values (k-step m of lane half hh covers k = 16 m + 8 hh + 0..7).
template <int D>
__global__ __launch_bounds__(kThreads) void dense_fwd_kernel(const float* __restrict__ H,
                                                             const float* __restrict__ W, int d_out,
                                                             float slope, int64_t N,
                                                             float* __restrict__ E_out,
                                                             uint8_t* __restrict__ mask) {
  constexpr int LD = D + 4, LPR = D / 4, TN = 64, NM = D / 16;
  const int DOP = (d_out + 31) & ~31, LDJ = DOP + 4, NOB = DOP / 32;
  float* H_s = reinterpret_cast<float*>(smem_raw);   // [TN][LD]
  float* J_s = H_s + TN * LD;                        // [TN][LDJ]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  const int ob = wave % NOB;                         // NOB <= 4 = waves
  const int rank = wave / NOB, sharers = (4 - ob + NOB - 1) / NOB;   // waves with this block: w = ob + NOB j
  Bf16Frag wh[NM], wm[NM], wl[NM];                   // pieces of W[ob * 32 + r][16 m + 8 hh + 0..7]
  {
    const int row = ob * 32 + r;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      float4 lo4 = make_float4(0.f, 0.f, 0.f, 0.f), hi4 = lo4;
      if (row < d_out) {
        lo4 = *reinterpret_cast<const float4*>(W + (size_t)row * D + 16 * m + 8 * hh);
        hi4 = *reinterpret_cast<const float4*>(W + (size_t)row * D + 16 * m + 8 * hh + 4);
      }
      const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
      split3x8(x, wh[m], wm[m], wl[m]);
    }
  }
  const int64_t n_tiles = (N + TN - 1) / TN;
  // the rows of the workgroup's next tile are requested while the current one is multiplied
  constexpr int CPT = TN * LPR / kThreads;
  float4 pre[CPT];
  auto load_tile = [&](int64_t tile) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int q = tid + k * kThreads;
      const int64_t n = tile * TN + q / LPR;
      pre[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (n < N) pre[k] = reinterpret_cast<const float4*>(H)[n * LPR + q % LPR];
    }
  };
  if (blockIdx.x < n_tiles) load_tile(blockIdx.x);
  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int64_t n0 = tile * TN;
    __syncthreads();   // previous tile's readers of H_s / J_s are done
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int q = tid + k * kThreads;
      *reinterpret_cast<float4*>(H_s + (q / LPR) * LD + (q % LPR) * 4) = pre[k];
    }
    if (tile + gridDim.x < n_tiles) load_tile(tile + gridDim.x);
    __syncthreads();
    for (int nb = rank; nb < 2; nb += sharers) {
      floatx16 acc = {0};
      const float* ap = H_s + (nb * 32 + r) * LD + hh * 8;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const float4 lo4 = *reinterpret_cast<const float4*>(ap + 16 * m), hi4 = *reinterpret_cast<const float4*>(ap + 16 * m + 4);
        const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        Bf16Frag ah, am, al;
        split3x8(x, ah, am, al);
        mfma_split(ah, am, al, wh[m], wm[m], wl[m], acc);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v)
        J_s[(nb * 32 + acc_row(v, lane)) * LDJ + ob * 32 + r] = acc[v];
    }
    __syncthreads();
    const int oc = d_out / 4;
    for (int q = tid; q < TN * oc; q += kThreads) {
      const int row = q / oc, c4 = q % oc;
      if (n0 + row < N) {
        float4 j = *reinterpret_cast<const float4*>(J_s + row * LDJ + c4 * 4);
        j.x = j.x > 0.f ? j.x : slope * j.x; j.y = j.y > 0.f ? j.y : slope * j.y;
        j.z = j.z > 0.f ? j.z : slope * j.z; j.w = j.w > 0.f ? j.w : slope * j.w;
        reinterpret_cast<float4*>(E_out)[(n0 + row) * oc + c4] = j;
      }
    }
    const int ob8 = d_out / 8;
    for (int q = tid; q < TN * ob8; q += kThreads) {
      const int row = q / ob8, b8 = q % ob8;
      if (n0 + row < N) {
        uint32_t bits = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) bits |= (J_s[row * LDJ + b8 * 8 + b] > 0.f ? 1u : 0u) << b;
        mask[(n0 + row) * ob8 + b8] = (uint8_t)bits;
      }
    }
  }
}

// grad_J = grad_E' * (mask ? 1 : slope); grad_H = grad_J W (also written to grad_E, which
// the edge stage then adds to); per-workgroup partial of grad_W = grad_J^T H_hat.
// deg_rowptr != nullptr (uniform layer): the copy in gH is divided by the row's out-degree.
// Eight waves at d = 128 (two per SIMD: one wave's LDS reads and stores overlap the other's
// products; a single resident workgroup has nothing else to overlap them with), four below.
template <int D>
constexpr int dense_bwd_waves() { return D == 128 ? 8 : 4; }

template <int D, int BITS>
__global__ __launch_bounds__(dense_bwd_waves<D>() * 64) void dense_bwd_kernel(Source srcH,
                                                             const uint8_t* __restrict__ mask,
                                                             const float* __restrict__ gEout,
                                                             const float* __restrict__ W, int d_out,
                                                             float slope, int64_t N,
                                                             float* gH,   // may be the buffer behind srcH
                                                             float* __restrict__ gE,
                                                             float* __restrict__ part_W,
                                                             double* __restrict__ zero_ptr,
                                                             int64_t zero_n,
                                                             const int32_t* __restrict__ deg_rowptr) {
  constexpr int LD = D + 4, LPR = D / 4, TN = 64, NIB = D / 32;
  constexpr int NWV = dense_bwd_waves<D>(), NT = NWV * 64;   // waves, threads
  constexpr int NWB = (4 * NIB + NWV - 1) / NWV;             // grad_W blocks per wave (at most 4 NIB blocks)
  // (the double-precision rows that the edge stage adds to start from zero: cleared here,
  // a launch earlier, instead of by a kernel of their own)
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < zero_n; i += (int64_t)gridDim.x * NT)
    zero_ptr[i] = 0.0;
  const int DOP = (d_out + 31) & ~31, LDJ = DOP + 4, NOB = DOP / 32;
  float* W_s = reinterpret_cast<float*>(smem_raw);   // [DOP][LD]
  float* Hh_s = W_s + DOP * LD;                      // [TN][LD]
  float* gJ_s = Hh_s + TN * LD;                      // [TN][LDJ]
  float* sc_s = gJ_s + TN * LDJ;                     // [TN] factor of the grad_H copy in gH (uniform layer: 1 / deg)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int q = tid; q < DOP * LPR; q += NT) {
    const int row = q / LPR, li = q % LPR;
    float4 w = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < d_out) w = reinterpret_cast<const float4*>(W)[row * LPR + li];
    *reinterpret_cast<float4*>(W_s + row * LD + li * 4) = w;
  }
  floatx16 accW[NWB];
#pragma unroll
  for (int j = 0; j < NWB; ++j) accW[j] = floatx16{0};

  const int64_t n_tiles = (N + TN - 1) / TN;
  const int ocp = DOP / 4, oc = d_out / 4;
  // the saved rows, upstream gradient and mask bits of the workgroup's next tile are
  // requested while the current one is multiplied (d_out <= 128: at most 8 chunks a thread)
  constexpr int CPT = TN * LPR / NT, GPT = TN * 32 / NT;
  RawChunk<BITS> preH[CPT];
  float4 preG[GPT];
  uint32_t preM[GPT];
  float preS = 1.f;
  auto load_tile = [&](int64_t tile) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int q = tid + k * NT;
      const int64_t n = tile * TN + q / LPR;
      preH[k].load(srcH, (n < N ? n : 0) * LPR + q % LPR);   // past the end: row 0, zeroed below
    }
    if (deg_rowptr && tid < TN) {
      // (uniform layer: the sparse stage gathers grad_H_h / deg(h); the division is done here, once per row)
      const int64_t n = tile * TN + tid;
      const int dg = n < N ? deg_rowptr[n + 1] - deg_rowptr[n] : 0;
      preS = dg > 0 ? 1.0f / (float)dg : 0.f;
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int q = tid + k * NT;
      const int64_t n = tile * TN + q / ocp;
      const int c4 = q % ocp;
      preG[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      preM[k] = 0u;
      if (q < TN * ocp && n < N && c4 < oc) {
        preG[k] = reinterpret_cast<const float4*>(gEout)[n * oc + c4];
        const int64_t bit = (n * oc + c4) * 4;
        preM[k] = (mask[bit >> 3] >> (bit & 7)) & 0xFu;
      }
    }
  };
  if (blockIdx.x < n_tiles) load_tile(blockIdx.x);
  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int64_t n0 = tile * TN;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int q = tid + k * NT;
      const int row = q / LPR;
      const float4 x = n0 + row < N ? preH[k].get() : make_float4(0.f, 0.f, 0.f, 0.f);
      *reinterpret_cast<float4*>(Hh_s + row * LD + (q % LPR) * 4) = x;
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int q = tid + k * NT;
      if (q < TN * ocp) {
        float4 g = preG[k];
        const uint32_t mb = preM[k];
        g.x *= (mb & 1u) ? 1.f : slope; g.y *= (mb & 2u) ? 1.f : slope;
        g.z *= (mb & 4u) ? 1.f : slope; g.w *= (mb & 8u) ? 1.f : slope;
        *reinterpret_cast<float4*>(gJ_s + (q / ocp) * LDJ + (q % ocp) * 4) = g;
      }
    }
    if (tid < TN) sc_s[tid] = preS;
    if (tile + gridDim.x < n_tiles) load_tile(tile + gridDim.x);
    __syncthreads();
    // grad_H tile: [n][i] = sum_o gJ[n][o] W[o][i]
    for (int blk = wave; blk < 2 * NIB; blk += NWV) {
      const int nb = blk & 1, ib = blk >> 1;
      floatx16 acc = {0};
      mfma_block<KCONT, KMAJOR>(gJ_s + nb * 32 * LDJ, LDJ, W_s + ib * 32, LD, DOP, acc);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t n = n0 + nb * 32 + acc_row(v, lane);
        if (n < N) {
          gH[n * D + ib * 32 + (lane & 31)] = acc[v] * sc_s[nb * 32 + acc_row(v, lane)];
          gE[n * D + ib * 32 + (lane & 31)] = acc[v];
        }
      }
    }
    // grad_W partial: [o][i] += sum_n gJ[n][o] H_hat[n][i]
#pragma unroll
    for (int j = 0; j < NWB; ++j) {
      const int blk = wave + NWV * j;
      if (blk < NOB * NIB) {
        const int ob = blk / NIB, ib = blk % NIB;
        mfma_block<KMAJOR, KMAJOR>(gJ_s + ob * 32, LDJ, Hh_s + ib * 32, LD, TN, accW[j]);
      }
    }
  }
  float* out = part_W + (size_t)blockIdx.x * d_out * D;
#pragma unroll
  for (int j = 0; j < NWB; ++j) {
    const int blk = wave + NWV * j;
    if (blk < NOB * NIB) {
      const int ob = blk / NIB, ib = blk % NIB;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = ob * 32 + acc_row(v, lane);
        if (o < d_out) out[o * D + ib * 32 + (lane & 31)] = accW[j][v];
      }
    }
  }
}

// One reduction job: out[seg][j] = sum over p in [ptr[seg], ptr[seg+1]) of
// part[p * stride + j].  Fixed order: thread group k of 4 sums partials p0+k, p0+k+4, ... in
// double, the four group sums are then added in order 0..3.  seg_ptr == nullptr: one segment
// [0, n_single).  nx = ceil(stride / 64) blocks of 256 threads per segment (0: job unused).
struct ReduceJob {
  const float* part;
  const int32_t* seg_ptr;
  int n_single, stride, nx, ny;
  float* out;
};
// Folding the double-precision rows of the heavy nodes into grad_E (see GradSink below).
struct HeavyFinish {
  const double* heavy;
  const int32_t* node;
  int64_t n;        // n_acc_heavy * D (0: nothing to do)
  int D;
  float* gE;
};

__device__ __forceinline__ void reduce_job(const ReduceJob& job, int bx, int by, double (*red)[64]) {
  const int seg = by;
  const int p0 = job.seg_ptr ? job.seg_ptr[seg] : 0, p1 = job.seg_ptr ? job.seg_ptr[seg + 1] : job.n_single;
  const int stride = job.stride;
  const int j = bx * 64 + (threadIdx.x & 63), k = threadIdx.x >> 6;
  const float* part = job.part;
  double s = 0.0;
  if (j < stride) {
    int p = p0 + k;
    for (; p + 12 < p1; p += 16) {      // four loads in flight, added in the same order
      const float a = part[(size_t)p * stride + j], b = part[(size_t)(p + 4) * stride + j];
      const float c = part[(size_t)(p + 8) * stride + j], d = part[(size_t)(p + 12) * stride + j];
      s += (double)a; s += (double)b; s += (double)c; s += (double)d;
    }
    for (; p < p1; p += 4) s += (double)part[(size_t)p * stride + j];
  }
  red[k][threadIdx.x & 63] = s;
  __syncthreads();
  if (k == 0 && j < stride)
    job.out[(size_t)seg * stride + j] = (float)(((red[0][j & 63] + red[1][j & 63]) + red[2][j & 63]) + red[3][j & 63]);
}

// Where the edge stage adds its gradient rows.  grad_E itself (fp32, preset to grad_H,
// the e_h term of H_h = e_h + sum pi e_t) takes the rows of ordinary nodes with fp32
// atomics.  A node that receives more than kAccHeavyDegree rows -- a hot tail sums 10^5
// and more O(1) terms of both signs, which fp32 accumulation cannot hold to 1e-5 of the
// result -- has a row of doubles in the compact buffer `heavy` instead; the epilogue kernel
// folds that row into grad_E at the end.  A staged node id carries the choice in bit 30.
struct GradSink {
  float* gE;              // [n_nodes, D]
  double* heavy;          // [n_acc_heavy, kHeavyReplicas, D]
  const int32_t* slot;    // [n_nodes] row of `heavy`, or -1
};
constexpr int kHeavyBit = 0x40000000;
// Every heavy node has kHeavyReplicas rows; a workgroup adds to the replica picked by its
// index, which divides the number of atomics that queue up on one address (a node with
// 10^5 and more rows is hit by every workgroup).
constexpr int kHeavyReplicas = 16;

template <int D>
__device__ __forceinline__ void sink_add(const GradSink& sink, int flagged_node, int col, float v) {
  const int node = flagged_node & kNodeIdMask;
  if (flagged_node & kHeavyBit) {
    const int64_t row = (int64_t)sink.slot[node] * kHeavyReplicas + (blockIdx.x & (kHeavyReplicas - 1));
    unsafeAtomicAdd(sink.heavy + row * D + col, (double)v);
  } else {
    unsafeAtomicAdd(sink.gE + (int64_t)node * D + col, v);
  }
}

// grad_E rows of the nodes that accumulated in double: replicas summed in order, plus
// grad_H (already in grad_E), rounded once.
__device__ __forceinline__ void finish_heavy(const HeavyFinish& hf, int64_t first, int64_t stride) {
  for (int64_t i = first; i < hf.n; i += stride) {
    const int64_t q = i / hf.D, col = i % hf.D;
    double sum = 0.0;
    for (int k = 0; k < kHeavyReplicas; ++k) sum += hf.heavy[(q * kHeavyReplicas + k) * hf.D + col];
    float* dst = hf.gE + (int64_t)hf.node[q] * hf.D + col;
    *dst = (float)(sum + (double)*dst);
  }
}

// The end of a backward pass in ONE launch (each launch costs several microseconds of a
// step that takes about a millisecond): blockIdx.z picks the job -- up to three reductions
// of partial parameter gradients and the heavy-node rows.  Blocks outside a job's range exit.
__global__ __launch_bounds__(256) void epilogue_kernel(ReduceJob j0, ReduceJob j1, ReduceJob j2,
                                                       HeavyFinish hf) {
  __shared__ double red[4][64];
  const int z = blockIdx.z;
  if (z == 3) {
    if (blockIdx.y == 0)
      finish_heavy(hf, (int64_t)blockIdx.x * 256 + threadIdx.x, (int64_t)gridDim.x * 256);
    return;
  }
  const ReduceJob& job = z == 0 ? j0 : z == 1 ? j1 : j2;
  if ((int)blockIdx.x >= job.nx || (int)blockIdx.y >= job.ny) return;
  reduce_job(job, blockIdx.x, blockIdx.y, red);
}

// ---------------------------------------------- uniform attention, backward ----
// grad_E_t += grad_H_h / deg(h) over the in-edges (h -> t) of t: the transposed sparse
// product of Eq. (2)'s grad_E = ctx(A_hat, grad_H) for the row-normalised adjacency
// (pi = 1 / deg).  The dense stage has already divided the rows it hands over by deg(h), so an
// edge costs its two ids and one gathered row.  One wave per 32 consecutive edges of the
// graph's tail order (all in-edges of a tail are adjacent, heads ascending): rows of equal
// tails are summed in fp32 before one row leaves the wave per run.  A run that holds ALL
// in-edges of its tail (it neither continues from the previous tile nor into the next) is the
// only writer of that row and adds with a plain read-modify-write; runs cut by a tile
// boundary, and the tails that accumulate in double, use atomics.
__global__ void zero_f32_fill_kernel(float* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = 0.f;
}

// What one edge (h -> t) passes to its tail in the generic transposed walk below, column by
// column: a per-edge word staged once per row and the value of column c.
template <int D, typename ARG>
struct MaxRows {         // grad_M[h, c] where this edge is the one whose number the head saved
  const int32_t* rowptr;
  const int32_t* r_eid;
  const float* gM;
  const ARG* arg;
  __device__ __forceinline__ int stage(int h, int64_t pos) const { return r_eid[pos] - rowptr[h] + 1; }
  __device__ __forceinline__ float value(int word, int h, int c) const {   // rows past the end: word = 0
    const int64_t i = (int64_t)h * D + c;
    return (int)arg[i] + 1 == word ? gM[i] : 0.f;
  }
};

template <int D>
__global__ __launch_bounds__(kThreads) void uniform_tail_kernel(
    const int32_t* __restrict__ c_head, const int32_t* __restrict__ c_tail,
    const float* __restrict__ gHs, int64_t n_edges, GradSink sink) {
  constexpr int NQ = D >= 64 ? 1 : 64 / D, RP = 32 / NQ;   // row parts of a wave
  constexpr int CPL = D >= 64 ? D / 64 : 1;                // columns per lane
  __shared__ int tl_s[kThreads / 64][32];
  __shared__ int hd_s[kThreads / 64][32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 31;
  const int64_t pos0 = ((int64_t)blockIdx.x * (kThreads / 64) + wave) * 32;
  if (pos0 >= n_edges) return;
  const int nrow = (int)min((int64_t)32, n_edges - pos0);
  int t_id = kNodeIdMask, h = -1;                            // past the end: an id no node has, no row
  if (r < nrow) { h = c_head[pos0 + r]; t_id = c_tail[pos0 + r]; }
  // the tails next to the tile (bit 30 included, as in the tile's own ids); -1: none
  const int t_before = pos0 > 0 ? c_tail[pos0 - 1] : -1;
  const int t_after = pos0 + 32 < n_edges ? c_tail[pos0 + 32] : -1;
  const int t_next = __shfl_down(t_id, 1), t_prev = __shfl_up(t_id, 1);
  const bool live = r < nrow;
  const bool stop = r + 1 == nrow || (r + 1) % RP == 0;
  const bool ends = live && (stop || t_next != t_id);
  const bool starts = live && (r % RP == 0 || t_prev != t_id);
  const bool start_closed = r == 0 ? t_before != t_id : t_prev != t_id;
  const bool end_closed = r + 1 == nrow ? t_after != t_id : t_next != t_id;
  const uint32_t start_mask = (uint32_t)__ballot(starts);
  const uint32_t closed_mask = (uint32_t)__ballot(starts && start_closed);
  const uint32_t upto = r == 31 ? 0xffffffffu : ((2u << r) - 1u);
  const int first = 31 - __clz((int)(start_mask & upto));    // first row of the run that row r belongs to
  const bool alone = ends && end_closed && !(t_id & kHeavyBit) && first >= 0 && ((closed_mask >> first) & 1u);
  const uint32_t alone_mask = (uint32_t)__ballot(alone);   // rows whose flush is the row's only writer
  if (lane < 32) { tl_s[wave][r] = t_id | (ends ? (int)0x80000000 : 0); hd_s[wave][r] = h; }
  __builtin_amdgcn_wave_barrier();
  const int col = lane % (D >= 64 ? 64 : D), e0 = (D >= 64 ? 0 : lane / D) * RP;
#pragma unroll
  for (int cp = 0; cp < CPL; ++cp) {
    const int c = col + 64 * cp;
    int node[RP];
    float val[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) {
      node[k] = tl_s[wave][e0 + k];
      const int hk = hd_s[wave][e0 + k];
      val[k] = hk >= 0 ? gHs[(int64_t)hk * D + c] : 0.f;
    }
    float run = 0.f;
#pragma unroll
    for (int k = 0; k < RP; ++k) {
      run += val[k];
      if (node[k] < 0) {
        if ((alone_mask >> (e0 + k)) & 1u) {
          float* dst = sink.gE + (int64_t)(node[k] & kNodeIdMask) * D + c;
          *dst += run;
        } else {
          sink_add<D>(sink, node[k], c, run);
        }
        run = 0.f;
      }
    }
  }
}

template <int D, typename ROWS>
__global__ __launch_bounds__(kThreads) void uniform_bwd_kernel(
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const uint8_t* __restrict__ r_hperm, ROWS rows, int64_t n_edges, GradSink sink) {
  constexpr int NQ = D >= 64 ? 1 : 64 / D, RP = 32 / NQ;   // row parts of a wave
  constexpr int CPL = D >= 64 ? D / 64 : 1;                // columns per lane
  __shared__ int tl_s[kThreads / 64][32];
  __shared__ int hd_s[kThreads / 64][32];
  __shared__ int w_s[kThreads / 64][32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 31;
  const int64_t pos0 = ((int64_t)blockIdx.x * (kThreads / 64) + wave) * 32;
  if (pos0 >= n_edges) return;
  const int nrow = (int)min((int64_t)32, n_edges - pos0);
  int t_id = 0, h = 0, w = 0;
  if (r < nrow) {
    const int64_t pos = pos0 + r;
    h = r_head[pos];
    t_id = r_tail[pos] | ((r_hperm[pos] & 0x40) ? kHeavyBit : 0);
    w = rows.stage(h, pos);
  }
  const int t_next = __shfl_down(t_id, 1);
  const bool stop = r + 1 == nrow || (r + 1) % RP == 0;
  const int flag = (r < nrow && (stop || t_next != t_id)) ? (int)0x80000000 : 0;
  if (lane < 32) { tl_s[wave][r] = t_id | flag; hd_s[wave][r] = h; w_s[wave][r] = w; }
  __builtin_amdgcn_wave_barrier();
  const int col = lane % (D >= 64 ? 64 : D), e0 = (D >= 64 ? 0 : lane / D) * RP;
#pragma unroll
  for (int cp = 0; cp < CPL; ++cp) {
    const int c = col + 64 * cp;
    int node[RP];
    float val[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) {
      node[k] = tl_s[wave][e0 + k];
      val[k] = rows.value(w_s[wave][e0 + k], hd_s[wave][e0 + k], c);
    }
    float run = 0.f;
#pragma unroll
    for (int k = 0; k < RP; ++k) {
      run += val[k];
      if (node[k] < 0) {
        sink_add<D>(sink, node[k], c, run);
        run = 0.f;
      }
    }
  }
}

// ------------------------------------------------------- edge-level backward ----
// Cooperative form (d = 128: W_r alone takes 66 KiB of LDS, so one workgroup -- eight waves,
// two per SIMD -- fills a compute unit and all of them share one 32-edge tile).  Phases of a
// tile, separated by workgroup barriers, and who does what:
//   stage: rows (prefetched raw one tile ahead, node ids two tiles ahead), per-edge scalars
//          and scatter flags (first wave)
//   1:     waves 0-3: a for channel block w;  waves 4-7: b for channel block w - 4 (bf16
//          matrix cores, operands split on the fly), then grad_a = gs tanh(b) and
//          f = gs (1 - tanh(b)^2) to LDS
//   1':    waves 0-3: grad_b = a * f, in place in LDS
//   2:     Pt (waves 0-3) / Ph (waves 4-7) for one column block each; every wave two of the
//          sixteen grad_W_r blocks
//   3:     Pt, Ph back to LDS; flag-driven scatter (as in the wave-independent kernel below)
constexpr int kCoopWaves = 8;

template <int D, int TE, int BITS>
__global__ __launch_bounds__(kCoopWaves * 64) void edge_bwd_kernel(
    Source src, const float* __restrict__ Wr, const float* __restrict__ er,
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const int32_t* __restrict__ r_eid, const uint8_t* __restrict__ r_hperm, ChunkList chunks,
    const float* __restrict__ pi, const float* __restrict__ gs, const float* __restrict__ gH,
    GradSink sink, float* __restrict__ part_Wr, float* __restrict__ part_er) {
  static_assert(TE == 32 && D == 128, "eight waves: four channel blocks x {a, b}");
  constexpr int NT = kCoopWaves * 64;
  constexpr int LD = D + 4, LPR = D / 4, NIB = D / 32;
  constexpr int NBW = NIB * NIB / kCoopWaves;     // grad_W_r blocks per wave (2)
  constexpr int NQ = NT / D, RP = TE / NQ;        // scatter: row parts (4 x 8 rows)
  constexpr int CPT = TE * LPR / NT;              // row chunks per thread and matrix (2)
  constexpr int RSTEP = NT / LPR;                 // rows between a thread's chunks
  float* Wr_s = reinterpret_cast<float*>(smem_raw);
  float* Et_s = Wr_s + D * LD;
  float* Eh_s = Et_s + TE * LD;
  float* dA_s = Eh_s + TE * LD;
  float* dB_s = dA_s + TE * LD;
  float* er_s = dB_s + TE * LD;
  float* gs_s = er_s + D;
  float* pi_s = gs_s + TE;
  int* tl_s = reinterpret_cast<int*>(pi_s + TE);   // tail of row e; sign bit: a tail run ends here
  int* hd_s = tl_s + TE;                           // head of row e
  int* hp_s = hd_s + TE;                           // row of head-order rank k
  int* hr_s = hp_s + TE;                           // head of rank k; sign bit: a head run ends here
  // run form (a tile whose edges share one tail; see the wave-independent kernel below)
  float* S_s = reinterpret_cast<float*>(hr_s + TE);    // [D] sum_e grad_a_e
  float* Pt_s = S_s + D;                               // [D] S W_r
  int* flag_s = reinterpret_cast<int*>(Pt_s + D);      // [0]: the current tile has one tail

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ch = blockIdx.x;
  const int rel = chunks.rel[ch], start = chunks.start[ch], count = chunks.count[ch];
  const int row0 = tid / LPR, li = tid % LPR;     // this thread stages rows row0 + k * RSTEP
  const int blk4 = wave & 3;                      // channel / column block of this wave's products
  const bool b_side = wave >= 4;                  // waves 4-7: b and Ph; waves 0-3: a and Pt

  // prefetch: raw rows of the next tile, node ids of the tile after it
  int tn[CPT], hn[CPT];
  auto load_ids = [&](int t0) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int row = t0 + row0 + k * RSTEP;
      tn[k] = 0; hn[k] = 0;
      if (row < count) { tn[k] = r_tail[start + row]; hn[k] = r_head[start + row]; }
    }
  };
  RawChunk<BITS> rt[CPT], rh[CPT];
  auto load_rows = [&]() {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      rt[k].load(src, (int64_t)tn[k] * LPR + li);
      rh[k].load(src, (int64_t)hn[k] * LPR + li);
    }
  };
  // per-edge scalars of the tile, held by the first wave (lane l and l + 32: row l % 32)
  const int er_row = lane & 31;
  int t_nx = 0, h_nx = 0, e_nx = -1, hp_nx = 0;
  auto load_edge = [&](int t0) {
    t_nx = 0; h_nx = 0; e_nx = -1; hp_nx = 0;
    if (wave == 0 && t0 + er_row < count) {
      const int pos = start + t0 + er_row;
      t_nx = r_tail[pos]; h_nx = r_head[pos]; e_nx = r_eid[pos]; hp_nx = r_hperm[pos];
    }
  };
  float g_ld = 0.f, p_ld = 0.f;
  int t_ld = 0, h_ld = 0, hp_ld = 0;
  auto load_weights = [&]() {
    g_ld = 0.f; p_ld = 0.f;
    if (e_nx >= 0) { g_ld = gs[e_nx]; p_ld = pi[e_nx]; }
    t_ld = t_nx; h_ld = h_nx; hp_ld = hp_nx;
  };
  load_ids(0);
  load_edge(0);
  load_rows();
  load_weights();
  load_ids(TE);
  load_edge(TE);

  const float4* Wg = reinterpret_cast<const float4*>(Wr + (size_t)rel * D * D);
  for (int q = tid; q < D * LPR; q += NT)
    *reinterpret_cast<float4*>(Wr_s + (q / LPR) * LD + (q % LPR) * 4) = Wg[q];
  for (int c = tid; c < D; c += NT) er_s[c] = er[(size_t)rel * D + c];

  floatx16 accW[NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j) accW[j] = floatx16{0};
  float er_acc = 0.f;

  for (int t0 = 0; t0 < count; t0 += TE) {
    const int nrow = min(TE, count - t0);
    __syncthreads();   // previous tile's scatter has finished reading LDS
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int row = row0 + k * RSTEP;
      *reinterpret_cast<float4*>(Et_s + row * LD + li * 4) = rt[k].get();
      *reinterpret_cast<float4*>(Eh_s + row * LD + li * 4) = rh[k].get();
    }
    if (wave == 0) {
      // where the scatter flushes its running sums (see the wave-independent kernel)
      const int perm = hp_ld & 31;
      const int t_id = t_ld | ((hp_ld & 0x40) ? kHeavyBit : 0), h_id = h_ld | ((hp_ld & 0x80) ? kHeavyBit : 0);
      const int h_rank = __shfl(h_id, perm);
      const int t_next = __shfl_down(t_id, 1), h_next = __shfl_down(h_rank, 1);
      const bool stop = er_row + 1 == nrow || (er_row + 1) % RP == 0;
      const int t_flag = (er_row < nrow && (stop || t_next != t_id)) ? (int)0x80000000 : 0;
      const int h_flag = (er_row < nrow && (stop || h_next != h_rank)) ? (int)0x80000000 : 0;
      if (lane < 32) {
        gs_s[er_row] = g_ld; pi_s[er_row] = p_ld; hd_s[er_row] = h_ld; hp_s[er_row] = perm;
        tl_s[er_row] = t_id | t_flag; hr_s[er_row] = h_rank | h_flag;
      }
      const int one = __all(er_row >= nrow || t_ld == __builtin_amdgcn_readfirstlane(t_ld));
      if (lane == 0) flag_s[0] = one;
    }
    if (t0 + TE < count) {
      load_rows();
      load_weights();
      load_ids(t0 + 2 * TE);
      load_edge(t0 + 2 * TE);
    }
    __syncthreads();
    const bool one_tail = flag_s[0] != 0;          // the same for the whole workgroup
    // ---- 1. a (waves 0-3) or b (waves 4-7) of channel block blk4: [c][e], lane = edge
    //      on the bf16 matrix cores: both operands are read as fp32, eight k-values at a time,
    //      and split into their three bfloat16 pieces in registers (see split3x8)
    floatx16 acc1 = {0};
    {
      const float* wrow = Wr_s + (blk4 * 32 + (lane & 31)) * LD + (lane >> 5) * 8;
      const float* xrow = (b_side ? Eh_s : Et_s) + (lane & 31) * LD + (lane >> 5) * 8;
      auto frag = [](const float* p, Bf16Frag& h, Bf16Frag& m, Bf16Frag& l) {
        const float4 lo4 = *reinterpret_cast<const float4*>(p), hi4 = *reinterpret_cast<const float4*>(p + 4);
        const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        split3x8(x, h, m, l);
      };
#pragma unroll
      for (int m = 0; m < D / 16; ++m) {
        Bf16Frag wh, wm, wl, xh, xm, xl;
        frag(wrow + 16 * m, wh, wm, wl);
        frag(xrow + 16 * m, xh, xm, xl);
        mfma_split(wh, wm, wl, xh, xm, xl, acc1);
      }
    }
    const int e1 = lane & 31;
    if (b_side) {
      const float g = gs_s[e1];
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int c0 = blk4 * 32 + 8 * vg + 4 * (lane >> 5);
        float da[4], f[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float vv = tanh_rel(acc1[4 * vg + u] + er_s[c0 + u]);
          da[u] = g * vv;
          f[u] = g * (1.f - vv * vv);
        }
        *reinterpret_cast<float4*>(dA_s + e1 * LD + c0) = make_float4(da[0], da[1], da[2], da[3]);
        *reinterpret_cast<float4*>(dB_s + e1 * LD + c0) = make_float4(f[0], f[1], f[2], f[3]);
        if (one_tail) {        // S: grad_a summed over the tile's 32 edges (the lanes of a half)
#pragma unroll
          for (int u = 0; u < 4; ++u) da[u] = slot_sum<32>(da[u]);
          if (e1 == 0) *reinterpret_cast<float4*>(S_s + c0) = make_float4(da[0], da[1], da[2], da[3]);
        }
      }
    }
    __syncthreads();
    // ---- 1'. grad_b = a * f (the wave that holds a; each element is its own)
    if (!b_side) {
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int c0 = blk4 * 32 + 8 * vg + 4 * (lane >> 5);
        float4 f = *reinterpret_cast<const float4*>(dB_s + e1 * LD + c0);
        f.x *= acc1[4 * vg + 0]; f.y *= acc1[4 * vg + 1]; f.z *= acc1[4 * vg + 2]; f.w *= acc1[4 * vg + 3];
        *reinterpret_cast<float4*>(dB_s + e1 * LD + c0) = f;
      }
    }
    __syncthreads();
    if (tid < D) {
      float sum = 0.f;
#pragma unroll 8
      for (int e = 0; e < TE; ++e) sum += dB_s[e * LD + tid];
      er_acc += sum;
    }
    // grad_H rows of the tile's heads (the e_t term of H_h): requested before the products
    const int si = tid % D, se0 = (tid / D) * RP;   // scatter: this thread's column and rows
    float ghv[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) ghv[k] = gH[(int64_t)hd_s[se0 + k] * D + si];
    // ---- 2. Pt = grad_a W_r (waves 0-3) or Ph = grad_b W_r (waves 4-7), column block blk4
    //      (run form: Pt is the one row S W_r; half hh of the wave sums half of the channels)
    floatx16 accP = {0};
    const bool run_form = one_tail && !b_side;
    if (run_form) {
      float p = 0.f;
      const float* wcol = Wr_s + (lane >> 5) * (D / 2) * LD + blk4 * 32 + (lane & 31);
      const float* sp = S_s + (lane >> 5) * (D / 2);
#pragma unroll 4
      for (int c = 0; c < D / 2; c += 4) {
        const float4 s4 = *reinterpret_cast<const float4*>(sp + c);
        p = fmaf(s4.x, wcol[c * LD], p);
        p = fmaf(s4.y, wcol[(c + 1) * LD], p);
        p = fmaf(s4.z, wcol[(c + 2) * LD], p);
        p = fmaf(s4.w, wcol[(c + 3) * LD], p);
      }
      p += __shfl_xor(p, 32);
      if (lane < 32) Pt_s[blk4 * 32 + lane] = p;
    } else {
      mfma_block<KCONT, KMAJOR>(b_side ? dB_s : dA_s, LD, Wr_s + blk4 * 32, LD, D, accP);
    }
    // grad_W_r blocks [c][i] += sum_e grad_a[e][c] e_t[e][i] + grad_b[e][c] e_h[e][i]
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
      const int blk = wave * NBW + j, cb = blk / NIB, ib = blk % NIB;
      // two-level sum: a fresh accumulator per tile, added to the chunk's accumulator
      // (keeps the fp32 running sum short when a relation has 10^5 and more edges)
      floatx16 accT = {0};
      if (one_tail) {          // S e_t^T: e_t is any row of the tile
        const float et = Et_s[ib * 32 + (lane & 31)];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 s4 = *reinterpret_cast<const float4*>(S_s + cb * 32 + 8 * q + 4 * (lane >> 5));
          accT[4 * q] = s4.x * et; accT[4 * q + 1] = s4.y * et; accT[4 * q + 2] = s4.z * et; accT[4 * q + 3] = s4.w * et;
        }
      } else {
        mfma_block<KMAJOR, KMAJOR>(dA_s + cb * 32, LD, Et_s + ib * 32, LD, TE, accT);
      }
      mfma_block<KMAJOR, KMAJOR>(dB_s + cb * 32, LD, Eh_s + ib * 32, LD, TE, accT);
      accW[j] += accT;
    }
    __syncthreads();   // every read of Et_s / Eh_s is done: reuse them as staging
    if (!run_form) {
      float* P_s = b_side ? Eh_s : Et_s;
#pragma unroll
      for (int v = 0; v < 16; ++v) P_s[acc_row(v, lane) * LD + blk4 * 32 + (lane & 31)] = accP[v];
    }
    __syncthreads();
    // scatter: every LDS read is independent of the running sums; a run inside a tile is
    // summed in fp32 and leaves as one atomic per column.  Rows past the end of the chunk
    // carry exact zeros (their weights gs, pi are 0) and no flag.
#pragma unroll
    for (int side = 0; side < 2; ++side) {
      int node[RP];
      float val[RP];
#pragma unroll
      for (int k = 0; k < RP; ++k) {
        if (side == 0) {
          node[k] = tl_s[se0 + k];
          // (run form: the whole tile is one run, whose product enters with its first row)
          const float pv = one_tail ? (se0 + k == 0 ? Pt_s[si] : 0.f) : Et_s[(se0 + k) * LD + si];
          val[k] = fmaf(pi_s[se0 + k], ghv[k], pv);
        } else {
          node[k] = hr_s[se0 + k];
          val[k] = Eh_s[hp_s[se0 + k] * LD + si];
        }
      }
      float run = 0.f;
#pragma unroll
      for (int k = 0; k < RP; ++k) {
        run += val[k];
        if (node[k] < 0) {
          sink_add<D>(sink, node[k], si, run);
          run = 0.f;
        }
      }
    }
  }
  float* outW = part_Wr + (size_t)ch * D * D;
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    const int blk = wave * NBW + j, cb = blk / NIB, ib = blk % NIB;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      outW[(cb * 32 + acc_row(v, lane)) * D + ib * 32 + (lane & 31)] = accW[j][v];
  }
  if (tid < D) part_er[(size_t)ch * D + tid] = er_acc;
}

// ------------------------------- edge-level backward, wave-independent form ----
// D = 32 or 64.  A workgroup of eight waves shares only W_r and e_r; every wave owns
// 32-edge tiles of the chunk end to end, with two wave-private LDS buffers X, Y of
// [32][D+4] floats that are reused three times per tile:
//   1. X, Y <- e_hat_t, e_hat_h rows (also kept in registers as MFMA operands)
//      a^T, b^T [e][c] = rows x W_r^T            (operands: registers x W_r in LDS)
//      grad_a, grad_b in place; grad_e_r column sums stay inside a lane
//      grad_W_r[c][i] += grad_a^T e_t + grad_b^T e_h   (registers x X, Y)
//   2. X, Y <- grad_a, grad_b
//      Pt, Ph [e][i] = grad_a W_r, grad_b W_r    (X, Y x W_r in LDS)
//   3. X, Y <- Pt, Ph; rows walked in tail order / head order, equal neighbours summed
//      in fp32, one atomic per run and column (fp64 for the rows of heavy nodes).
// Run form: the relation order is sorted by tail, so popular tails own long runs and more than
// half of the tiles of a Zipf-tailed graph hold ONE tail.  For such a tile the tail-side
// products depend on the edges only through S = sum_e grad_a_e: grad_W_r += S e_t^T (a rank-one
// update on the vector unit) and Pt = S W_r (one row, added with the tile's first row), so two
// of the six products -- half of the fp32 ones -- are skipped.  The host balances the
// workgroups' spans by tile cost, not by edge count.
// The transposed form of step 1 (edge index on the accumulator rows, channel on the
// lanes) is what lets grad_a / grad_b feed the grad_W_r products without leaving the
// registers.  There is no workgroup barrier between staging W_r and the final fixed-order
// combination of the eight waves' grad_W_r / grad_e_r partial sums.
constexpr int kEdgeWaves = 8;

template <int D>
constexpr int edge_wave_region() { return 2 * 32 * (D + 4) + 6 * 32; }   // floats per wave

// Phase boundary inside a wave that passes data between its lanes through LDS: the
// LDS queue of a wave is in order, so no hardware wait is needed; the compiler must
// only keep the phases apart (which also bounds how many loads it hoists at once).
__device__ __forceinline__ void phase_fence() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// One span (a run of whole chunks of one relation) by one workgroup; `ch` numbers the span and
// its slot in the partial-sum buffers.
template <int D, int BITS>
__device__ __forceinline__ void edge_wave_span(
    const int ch, const Source& src, const float* __restrict__ Wr, const float* __restrict__ er,
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const int32_t* __restrict__ r_eid, const uint8_t* __restrict__ r_hperm, const ChunkList& chunks,
    const float* __restrict__ pi, const float* __restrict__ gs, const float* __restrict__ gH,
    const GradSink& sink, float* __restrict__ part_Wr, float* __restrict__ part_er) {
  constexpr int LD = D + 4, LPR = D / 4, KH = D / 2, NB = D / 32, NW = kEdgeWaves;
  constexpr int NT = NW * 64, BUF = 32 * LD, REGION = edge_wave_region<D>();
  constexpr int NQ = 64 / D, RP = 32 / NQ;        // scatter: row parts of a wave
  float* Wr_s = reinterpret_cast<float*>(smem_raw);
  float* er_s = Wr_s + D * LD;
  float* regions = er_s + D;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* X_s = regions + wave * REGION;
  float* Y_s = X_s + BUF;
  float* gs_s = Y_s + BUF;
  float* pi_s = gs_s + 32;
  int* tl_s = reinterpret_cast<int*>(pi_s + 32);   // tail of row e; sign bit: a tail run ends here
  int* hd_s = tl_s + 32;                           // head of row e
  int* hp_s = hd_s + 32;                           // row of head-order rank k
  int* hr_s = hp_s + 32;                           // head of rank k; sign bit: a head run ends here

  const int rel = chunks.rel[ch], start = chunks.start[ch], count = chunks.count[ch];
  const int r = lane & 31, hh = lane >> 5;
  const int n_wt = (count + 31) >> 5;
  int wt = wave;

  int t_nx = 0, h_nx = 0, e_nx = -1, hp_nx = 0;
  auto load_idx = [&](int tile) {
    const int row = tile * 32 + r;
    t_nx = 0; h_nx = 0; e_nx = -1; hp_nx = 0;   // past the end: node 0 (a valid row), weight 0
    if (row < count) {
      const int pos = start + row;
      t_nx = r_tail[pos]; h_nx = r_head[pos]; e_nx = r_eid[pos]; hp_nx = r_hperm[pos];
    }
  };
  HalfRow<D, BITS> nt, nh;
  float g_ld = 0.f, p_ld = 0.f;
  int t_ld = 0, h_ld = 0, hp_ld = 0;
  auto load_rows = [&]() {
    nt.load(src, t_nx, hh);
    nh.load(src, h_nx, hh);
    g_ld = 0.f; p_ld = 0.f;
    if (e_nx >= 0) { g_ld = gs[e_nx]; p_ld = pi[e_nx]; }
    t_ld = t_nx; h_ld = h_nx; hp_ld = hp_nx;
  };

  const float4* Wg = reinterpret_cast<const float4*>(Wr + (size_t)rel * D * D);
  for (int q = tid; q < D * LPR; q += NT)
    *reinterpret_cast<float4*>(Wr_s + (q / LPR) * LD + (q % LPR) * 4) = Wg[q];
  for (int c = tid; c < D; c += NT) er_s[c] = er[(size_t)rel * D + c];
  __syncthreads();

  float er_c[NB], er_acc[NB];
#pragma unroll
  for (int cb = 0; cb < NB; ++cb) { er_c[cb] = er_s[cb * 32 + r]; er_acc[cb] = 0.f; }
  floatx16 accW[NB * NB];
#pragma unroll
  for (int j = 0; j < NB * NB; ++j) accW[j] = floatx16{0};

  for (; wt < n_wt; wt += NW) {
    // (fetching the next tile's rows a tile ahead gained nothing once the workgroups became
    // persistent -- the second wave of the SIMD covers the latency -- and cost INT8 rows 16 %
    // through the registers the raw words occupy)
    load_idx(wt);
    load_rows();
    const int nrow = min(32, count - wt * 32);
    // Rows are in tail order inside a relation, and popular tails own long runs: a tile whose
    // edges all share ONE tail needs W_r^T (sum_e grad_a_e) once, not W_r^T grad_a_e per edge.
    const bool one_tail = __all(r >= nrow || t_ld == __builtin_amdgcn_readfirstlane(t_ld)) != 0;
    {
      // where the scatter has to flush its running sums: at the last row of a run of
      // equal tails (rows are in tail order) resp. equal heads (ranks are in head order),
      // at the end of a lane's row part and at the tile's last row
      // (bit 30 of a staged id: the node accumulates in double -- bits 6, 7 of the row's byte)
      const int perm = hp_ld & 31;
      const int t_id = t_ld | ((hp_ld & 0x40) ? kHeavyBit : 0), h_id = h_ld | ((hp_ld & 0x80) ? kHeavyBit : 0);
      const int h_rank = __shfl(h_id, perm);                    // head of rank r
      const int t_next = __shfl_down(t_id, 1), h_next = __shfl_down(h_rank, 1);
      const bool stop = r + 1 == nrow || (r + 1) % RP == 0;
      const int t_flag = (r < nrow && (stop || t_next != t_id)) ? (int)0x80000000 : 0;
      const int h_flag = (r < nrow && (stop || h_next != h_rank)) ? (int)0x80000000 : 0;
      if (hh == 0) {
        gs_s[r] = g_ld; pi_s[r] = p_ld; hd_s[r] = h_ld; hp_s[r] = perm;
        tl_s[r] = t_id | t_flag; hr_s[r] = h_rank | h_flag;
      }
    }
#pragma unroll
    for (int i = 0; i < KH; i += 4) {
      *reinterpret_cast<float4*>(X_s + r * LD + hh * KH + i) =
          make_float4(nt.get(i), nt.get(i + 1), nt.get(i + 2), nt.get(i + 3));
      *reinterpret_cast<float4*>(Y_s + r * LD + hh * KH + i) =
          make_float4(nh.get(i), nh.get(i + 1), nh.get(i + 2), nh.get(i + 3));
    }
    phase_fence();

    // ---- 1a. a^T, b^T: accumulator row = edge, lane column = channel
    floatx16 accA[NB], accB[NB];
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) { accA[cb] = floatx16{0}; accB[cb] = floatx16{0}; }
    {
      // on the bf16 matrix cores: eight k-values of each operand are read as fp32, split into
      // three bfloat16 pieces in registers and multiplied piece by piece (see split3x8); the
      // W_r fragments serve both products and the row fragments both channel blocks, which is
      // what makes splitting on the fly pay here (it does not for the other two product pairs
      // of this kernel, whose fragments are used once)
      int wofs = 0;
      asm volatile("" : "+v"(wofs));    // W_r is re-read from LDS, never parked in registers
      const float* wrow = Wr_s + r * LD + hh * KH + wofs;
      const float* trow = X_s + r * LD + hh * KH + wofs;
      const float* hrow = Y_s + r * LD + hh * KH + wofs;
      auto frag = [](const float* p, Bf16Frag& h, Bf16Frag& m, Bf16Frag& l) {
        const float4 lo4 = *reinterpret_cast<const float4*>(p), hi4 = *reinterpret_cast<const float4*>(p + 4);
        const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        split3x8(x, h, m, l);
      };
#pragma unroll
      for (int m = 0; m < KH / 8; ++m) {
        Bf16Frag th, tm, tl, hhi, hmi, hlo, wh[NB], wm[NB], wl[NB];
        frag(trow + 8 * m, th, tm, tl);
        frag(hrow + 8 * m, hhi, hmi, hlo);
#pragma unroll
        for (int cb = 0; cb < NB; ++cb) frag(wrow + cb * 32 * LD + 8 * m, wh[cb], wm[cb], wl[cb]);
#define TINYKG_SPLIT_STEP(TP, HP, WP)                                                                      \
        _Pragma("unroll") for (int cb = 0; cb < NB; ++cb) {                                                \
          accA[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TP.v, WP[cb].v, accA[cb], 0, 0, 0);           \
          accB[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(HP.v, WP[cb].v, accB[cb], 0, 0, 0);           \
        }
        TINYKG_SPLIT_STEP(th, hhi, wl)
        TINYKG_SPLIT_STEP(tl, hlo, wh)
        TINYKG_SPLIT_STEP(tm, hmi, wm)
        TINYKG_SPLIT_STEP(th, hhi, wm)
        TINYKG_SPLIT_STEP(tm, hmi, wh)
        TINYKG_SPLIT_STEP(th, hhi, wh)
#undef TINYKG_SPLIT_STEP
        __builtin_amdgcn_sched_barrier(0);   // one k-step's fragments at a time
      }
    }
    phase_fence();
    // ---- 1b. grad_a = gs tanh(b), grad_b = gs a (1 - tanh(b)^2), in place
    {
      float er_t[NB];
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) er_t[cb] = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 g4 = *reinterpret_cast<const float4*>(gs_s + 8 * q + 4 * hh);   // edges of registers 4q..4q+3
        const float gq[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
          for (int cb = 0; cb < NB; ++cb) {
            const float vv = tanh_rel(accB[cb][4 * q + u] + er_c[cb]);
            const float db = gq[u] * accA[cb][4 * q + u] * (1.f - vv * vv);
            accA[cb][4 * q + u] = gq[u] * vv;
            accB[cb][4 * q + u] = db;
            er_t[cb] += db;
          }
        }
      }
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) er_acc[cb] += er_t[cb];
    }
    float s_col[NB];     // one_tail: S = sum_e grad_a_e, channel cb * 32 + r (both halves of the wave)
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      float t = 0.f;
      if (one_tail) {
#pragma unroll
        for (int v = 0; v < 16; ++v) t += accA[cb][v];
        t += __shfl_xor(t, 32);
      }
      s_col[cb] = t;
    }
    phase_fence();
    // ---- 1c. grad_W_r[c][i] += sum_e grad_a[e][c] e_t[e][i] + grad_b[e][c] e_h[e][i]
    //      (one_tail: the first sum is the rank-one matrix S e_t^T, added after the loop)
    //      (two-level sum: a fresh accumulator per tile keeps the fp32 running sum short)
    //      The operands of four accumulator registers (eight edges) are fetched from LDS
    //      while the products of the previous four run; the scheduling fences keep the
    //      compiler from fetching all of them at once, which would not fit the registers.
#pragma unroll
    for (int ib = 0; ib < NB; ++ib) {
      floatx16 accT[NB];
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) accT[cb] = floatx16{0};
      float bt[2][4], bh[2][4];
      auto fetch = [&](int q, float* t4, float* h4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = u + 8 * q + 4 * hh;          // = acc_row(4 q + u, lane)
          t4[u] = X_s[e * LD + ib * 32 + r];
          h4[u] = Y_s[e * LD + ib * 32 + r];
        }
      };
      fetch(0, bt[0], bh[0]);
      if (one_tail) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (q < 3) fetch(q + 1, bt[(q + 1) & 1], bh[(q + 1) & 1]);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int cb = 0; cb < NB; ++cb)
              accT[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(accB[cb][4 * q + u], bh[q & 1][u], accT[cb], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (q < 3) fetch(q + 1, bt[(q + 1) & 1], bh[(q + 1) & 1]);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int cb = 0; cb < NB; ++cb) {
              accT[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(accA[cb][4 * q + u], bt[q & 1][u], accT[cb], 0, 0, 0);
              accT[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(accB[cb][4 * q + u], bh[q & 1][u], accT[cb], 0, 0, 0);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) {
        accW[cb * NB + ib] += accT[cb];
        // pins the addition here: sunk to the end of the loop body it would keep the
        // tile's accumulators alive through the scatter
        asm volatile("" : "+v"(accW[cb * NB + ib]));
      }
    }
    if (one_tail) {
      // S e_t^T: row c of block cb needs S[c], which lane c % 32 holds; e_t is any row of X
      float et[NB];
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) et[ib] = X_s[ib * 32 + r];
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float sr = __shfl(s_col[cb], acc_row(v, lane));
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) accW[cb * NB + ib][v] = fmaf(sr, et[ib], accW[cb * NB + ib][v]);
        }
      }
    }
    phase_fence();
    // ---- 2. X, Y <- grad_a, grad_b as [e][c]
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int e = acc_row(v, lane);
        if (!one_tail) X_s[e * LD + cb * 32 + r] = accA[cb][v];   // (the run form works from S alone)
        Y_s[e * LD + cb * 32 + r] = accB[cb][v];
      }
    }
    // grad_H rows of the tile's heads (the e_t term of H_h): requested here so that they
    // arrive while the next products run
    const int si = lane % D, se0 = (lane / D) * RP;   // scatter: this lane's column and rows
    float ghv[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) {
      const int hk = D == 64 ? __builtin_amdgcn_readfirstlane(hd_s[se0 + k]) : hd_s[se0 + k];   // uniform when a row is a wave
      ghv[k] = gH[(int64_t)hk * D + si];
    }
    // P[e][i] = sum_c G[e][c] W_r[c][i] for G = grad_a (tails), then grad_b (heads); half hh
    // walks c = (s&7) + 16 (s>>3) + 8 hh, which keeps the two halves of a W_r read in
    // different LDS banks.  Then P goes back to the same buffer as [e][i] and its rows are
    // walked in tail order resp. head order: every LDS read is independent of the running
    // sum, a run inside a tile has at most 32 terms and is summed in fp32, and one
    // atomic per run and column leaves the wave.  Rows past the end of the chunk carry
    // exact zeros (their weights gs, pi are 0) and no flag.
#pragma unroll
    for (int side = 0; side < 2; ++side) {
      float* P_s = side == 0 ? X_s : Y_s;
      phase_fence();
      const bool run_form = side == 0 && one_tail;
      float pt_run = 0.f;                          // run_form: (sum_e grad_a_e) W_r, column si
      if (run_form) {
#pragma unroll
        for (int cb = 0; cb < NB; ++cb) {
#pragma unroll
          for (int j = 0; j < 32; ++j) {
            const float sc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s_col[cb]), j));
            pt_run = fmaf(sc, Wr_s[(cb * 32 + j) * LD + si], pt_run);
          }
        }
      } else {
      floatx16 accP[NB];
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) accP[ib] = floatx16{0};
      {
        int wofs = 0;
        asm volatile("" : "+v"(wofs));
        const float* wcol = Wr_s + r + wofs;
#pragma unroll
        for (int s0 = 0; s0 < KH; s0 += 4) {
          const int c0 = (s0 & 7) + 16 * (s0 >> 3) + 8 * hh;
          const float4 a4 = *reinterpret_cast<const float4*>(P_s + r * LD + c0);
          const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int ib = 0; ib < NB; ++ib)
              accP[ib] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], wcol[(c0 + u) * LD + ib * 32], accP[ib], 0, 0, 0);
          }
        }
      }
      phase_fence();
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
        for (int v = 0; v < 16; ++v) P_s[acc_row(v, lane) * LD + ib * 32 + r] = accP[ib][v];
      }
      }
      phase_fence();
      constexpr int RB = RP < 16 ? RP : 16;        // rows whose LDS reads are issued together
      float run = 0.f;
#pragma unroll
      for (int k0 = 0; k0 < RP; k0 += RB) {
        int node[RB];
        float val[RB];
#pragma unroll
        for (int k = 0; k < RB; ++k) {
          if (side == 0) {
            node[k] = tl_s[se0 + k0 + k];
            // (run_form: the whole tile is one run, whose product enters with its first row)
            const float pv = run_form ? (se0 + k0 + k == 0 ? pt_run : 0.f) : P_s[(se0 + k0 + k) * LD + si];
            val[k] = fmaf(pi_s[se0 + k0 + k], ghv[k0 + k], pv);
          } else {
            node[k] = hr_s[se0 + k0 + k];
            const int pk = D == 64 ? __builtin_amdgcn_readfirstlane(hp_s[se0 + k0 + k]) : hp_s[se0 + k0 + k];
            val[k] = P_s[pk * LD + si];
          }
        }
#pragma unroll
        for (int k = 0; k < RB; ++k) {
          run += val[k];
          // (D == 64: the row's node is the same in every lane; as a scalar it keeps the
          // address arithmetic and the heavy-node lookup off the vector unit)
          const int nk = D == 64 ? __builtin_amdgcn_readfirstlane(node[k]) : node[k];
          if (nk < 0) {
            sink_add<D>(sink, nk, si, run);
            run = 0.f;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    phase_fence();   // the next tile overwrites X, Y and the index arrays
  }

  // fixed-order combination of the eight waves' partial sums
  {
    float* mine = regions + wave * REGION;
#pragma unroll
    for (int j = 0; j < NB * NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) mine[(j * 16 + v) * 64 + lane] = accW[j][v];
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      const float both = er_acc[cb] + __shfl_xor(er_acc[cb], 32);
      if (hh == 0) mine[NB * NB * 1024 + cb * 32 + r] = both;
    }
  }
  __syncthreads();
  float* outW = part_Wr + (size_t)ch * D * D;
  for (int f = tid; f < D * D; f += NT) {
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += regions[w * REGION + f];
    const int l = f & 63, v = (f >> 6) & 15, j = f >> 10;
    const int cb = j / NB, ib = j % NB;
    outW[(cb * 32 + acc_row(v, l)) * D + ib * 32 + (l & 31)] = sum;
  }
  if (tid < D) {
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += regions[w * REGION + NB * NB * 1024 + tid];
    part_er[(size_t)ch * D + tid] = sum;
  }
}

// The persistent form: workgroup w walks the spans [group_ptr[w], group_ptr[w + 1]) -- its
// share of the relation order, about n_edges / gridDim.x edges -- so W_r is staged and the
// waves' partial parameter gradients are combined once per span (one or two per workgroup)
// instead of once per 500-edge chunk, and no workgroup is left over for a last round.
template <int D, int BITS>
__global__ __launch_bounds__(kEdgeWaves * 64) void edge_wave_kernel(
    Source src, const float* __restrict__ Wr, const float* __restrict__ er,
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const int32_t* __restrict__ r_eid, const uint8_t* __restrict__ r_hperm, ChunkList spans,
    const int32_t* __restrict__ group_ptr, const float* __restrict__ pi, const float* __restrict__ gs,
    const float* __restrict__ gH, GradSink sink, float* __restrict__ part_Wr, float* __restrict__ part_er) {
  const int first = group_ptr[blockIdx.x], last = group_ptr[blockIdx.x + 1];
  for (int sp = first; sp < last; ++sp) {
    if (sp != first) __syncthreads();   // the previous span's combination has read the waves' LDS regions
    edge_wave_span<D, BITS>(sp, src, Wr, er, r_head, r_tail, r_eid, r_hperm, spans, pi, gs, gH, sink, part_Wr, part_er);
  }
}

// ---------------------------------------------- edge-level backward, code form ----
// The d <= 64 edge kernel for a compressed context whose quantisation group covers at least a
// row (every row then has ONE (Z, scale) pair), with ALL six products on the bf16 matrix cores:
//   1a  a, b: Eq. (4) is linear, W_r e_hat = scale (W_r code) + Z (W_r 1); the integer codes are
//       exact bfloat16 values, so each product is three piece products with the pieces of W_r
//       (split once per span into LDS), and the rows are neither dequantised nor split.  The
//       row fragments come straight from the registers the rows were fetched into.
//   1c  grad_W_r = sum_e grad[e] e_hat[e]^T = sum_e (scale_e grad[e]) code[e]^T + (sum_e mid_e grad[e]) 1^T:
//       the left operand is the accumulator of step 1 itself (lane = channel, registers =
//       edges: exactly the operand layout with the edges as contraction index), scaled and
//       split in registers; the codes are read column-wise from the tile's code matrix in LDS;
//       the rank-one part is a per-lane sum that joins the tile's own partial sum.  (The codes
//       are centred, code - B/2, and Z becomes the row's midpoint: see where they are packed.)
//   2   Pt = grad_a W_r, Ph = grad_b W_r: grad rows go through LDS once (they must change from
//       lane = channel to lane = edge), are split on the fly and meet the pieces of W_r^T (split
//       once per span into LDS as well): six piece products.  The two sides run one after the
//       other through ONE fp32 buffer that overlays the (by then dead) code matrices.
// LDS: pieces of W_r and of W_r^T (2 x 27 KiB at d = 64) and 10.3 KiB per wave.
// Everything else (flags, scatter, partial sums) as in the fp32 form below.
template <int D>
constexpr int edge_code_region_bytes() { return 2 * 32 * (D + 8) * 2 + 10 * 32 * 4; }
template <int D>
constexpr int edge_code_smem_bytes() {
  // pieces of W_r and W_r^T, row sums, e_r, the waves' regions -- or, at the end of a span, the
  // waves' partial grad_W_r (which overlay everything)
  constexpr int work = 2 * 3 * D * (D + 8) * 2 + 2 * D * 4 + kEdgeWaves * edge_code_region_bytes<D>();
  constexpr int comb = kEdgeWaves * ((D / 32) * (D / 32) * 1024 + D) * 4;
  return work > comb ? work : comb;
}

// W_r^T as three bf16 matrices: Wt[i][c] = W[c][i], rows padded like stage_split_matrix's.
template <int D>
__device__ __forceinline__ void stage_split_matrix_transposed(const float* __restrict__ W, uint16_t* __restrict__ Wt,
                                                              int tid, int n_threads) {
  constexpr int LDW = D + 8;
  for (int q = tid; q < D * D; q += n_threads) {
    const int c = q / D, i = q % D;              // coalesced reads of W, strided 2-byte writes
    const float x = W[q];
    const uint32_t hb = __float_as_uint(x) & 0xFFFF0000u;
    const float r1 = x - __uint_as_float(hb);
    const uint32_t mb = __float_as_uint(r1) & 0xFFFF0000u;
    const uint32_t lb = __float_as_uint(r1 - __uint_as_float(mb));
    Wt[i * LDW + c] = (uint16_t)(hb >> 16);
    Wt[D * LDW + i * LDW + c] = (uint16_t)(mb >> 16);
    Wt[2 * D * LDW + i * LDW + c] = (uint16_t)(lb >> 16);
  }
}

// Four consecutive rows of one column of a row-major matrix of 16-bit values in LDS, for each of
// 32 columns at once: lane l receives M[row0 + 0..3][col0 + l % 32].  `ld` in elements; row0 may
// differ between the two lane halves.  (The transposing LDS read: each group of sixteen lanes
// passes the addresses of the sixteen 8-byte pieces of its 4 x 16 block, lane p of the group that
// of row p / 4, piece p % 4, and lane i of the group receives column i.)
__device__ __forceinline__ uint2 lds_column4(const uint16_t* M, int ld, int row0, int col0, int lane) {
  typedef short short4v __attribute__((ext_vector_type(4)));
  const uint16_t* p = M + (row0 + ((lane & 15) >> 2)) * ld + col0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(p));
  union { short4v s; uint2 u; } cv;
  cv.s = v;
  return cv.u;
}

// Sum of the integer codes of a whole row, from the two lane halves that hold it.
template <int D, int BITS>
__device__ __forceinline__ float code_sum(const HalfRow<D, BITS>& h) {
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < HalfRow<D, BITS>::NW; ++k) {
    uint32_t w = h.w[k];
    if (BITS == 1) { sum += (uint32_t)__builtin_popcount(w); continue; }
    if (BITS == 2) w = (w & 0x33333333u) + ((w >> 2) & 0x33333333u);              // 4-bit sums of two codes
    if (BITS <= 4) w = (w & 0x0F0F0F0Fu) + ((w >> 4) & 0x0F0F0F0Fu);              // byte sums
    sum = __builtin_amdgcn_sad_u8(w, 0u, sum);
  }
  const float f = (float)sum;
  return f + __shfl_xor(f, 32);
}

template <int D, int BITS>
__device__ __forceinline__ void edge_code_span(
    const int ch, const Source& src, const float* __restrict__ Wr, const float* __restrict__ er,
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const int32_t* __restrict__ r_eid, const uint8_t* __restrict__ r_hperm, const ChunkList& chunks,
    const float* __restrict__ pi, const float* __restrict__ gs, const float* __restrict__ gH,
    const GradSink& sink, float* __restrict__ part_Wr, float* __restrict__ part_er) {
  constexpr int LD = D + 4, LDW = D + 8, KH = D / 2, NB = D / 32, NM = KH / 8, NW = kEdgeWaves;
  constexpr int NT = NW * 64, REGION = edge_code_region_bytes<D>();
  constexpr int NQ = 64 / D, RP = 32 / NQ;        // scatter: row parts of a wave
  uint16_t* Wp = reinterpret_cast<uint16_t*>(smem_raw);                 // [3][D][LDW]: W_r, k = i contiguous
  uint16_t* Wtp = Wp + 3 * D * LDW;                                     // [3][D][LDW]: W_r^T, k = c contiguous
  float* wsum_s = reinterpret_cast<float*>(Wtp + 3 * D * LDW);          // row sums of W_r
  float* er_s = wsum_s + D;
  unsigned char* regions = reinterpret_cast<unsigned char*>(er_s + D);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned char* mine = regions + wave * REGION;
  uint16_t* Ct_s = reinterpret_cast<uint16_t*>(mine);                   // [32][LDW] codes of the tail rows
  uint16_t* Ch_s = Ct_s + 32 * LDW;                                     // [32][LDW] codes of the head rows
  float* G_s = reinterpret_cast<float*>(mine);                          // [32][LD] fp32, overlays both (step 2)
  float* gs_s = reinterpret_cast<float*>(mine + 2 * 32 * LDW * 2);
  float* pi_s = gs_s + 32;
  float* zt_s = pi_s + 32;                         // (mid, scale) of the tail / head row of edge e
  float* st_s = zt_s + 32;
  float* zh_s = st_s + 32;
  float* sh_s = zh_s + 32;
  int* tl_s = reinterpret_cast<int*>(sh_s + 32);   // tail of row e; sign bit: a tail run ends here
  int* hd_s = tl_s + 32;                           // head of row e
  int* hp_s = hd_s + 32;                           // row of head-order rank k
  int* hr_s = hp_s + 32;                           // head of rank k; sign bit: a head run ends here
  static_assert(2 * 32 * LDW * 2 >= 32 * LD * 4, "the fp32 buffer must fit over the two code matrices");

  const int rel = chunks.rel[ch], start = chunks.start[ch], count = chunks.count[ch];
  const int r = lane & 31, hh = lane >> 5;
  const int n_wt = (count + 31) >> 5;

  stage_split_matrix<D>(Wr + (size_t)rel * D * D, Wp, tid, NT);
  stage_split_matrix_transposed<D>(Wr + (size_t)rel * D * D, Wtp, tid, NT);
  for (int c = tid; c < D; c += NT) {
    er_s[c] = er[(size_t)rel * D + c];
    const float4* row = reinterpret_cast<const float4*>(Wr + ((size_t)rel * D + c) * D);
    double sum = 0.0;
    for (int q = 0; q < D / 4; ++q) { const float4 w = row[q]; sum += (double)w.x + (double)w.y + (double)w.z + (double)w.w; }
    wsum_s[c] = (float)sum;
  }
  __syncthreads();

  float er_c[NB], ws_c[NB], er_acc[NB];
#pragma unroll
  for (int cb = 0; cb < NB; ++cb) { er_c[cb] = er_s[cb * 32 + r]; ws_c[cb] = wsum_s[cb * 32 + r]; er_acc[cb] = 0.f; }
  floatx16 accW[NB * NB];
#pragma unroll
  for (int j = 0; j < NB * NB; ++j) accW[j] = floatx16{0};

  // the ids of a wave's next tile are requested a tile ahead (four registers): one hop less in
  // the chain ids -> rows that every tile starts with
  int t_nx = 0, h_nx = 0, e_nx = -1, hp_nx = 0;
  auto load_idx = [&](int tile) {
    const int row = tile * 32 + r;
    t_nx = 0; h_nx = 0; e_nx = -1; hp_nx = 0;       // past the end: node 0 (a valid row), weight 0
    if (tile < n_wt && row < count) {
      const int pos = start + row;
      t_nx = r_tail[pos]; h_nx = r_head[pos]; e_nx = r_eid[pos]; hp_nx = r_hperm[pos];
    }
  };
  load_idx(wave);
  for (int wt = wave; wt < n_wt; wt += NW) {
    // ---- stage: ids, flags, per-edge scalars; rows fetched as raw codes
    const int t_ld = t_nx, h_ld = h_nx, e_ld = e_nx, hp_ld = hp_nx;
    HalfRow<D, BITS> nt, nh;
    nt.load(src, t_ld, hh);
    nh.load(src, h_ld, hh);
    float g_ld = 0.f, p_ld = 0.f;
    if (e_ld >= 0) { g_ld = gs[e_ld]; p_ld = pi[e_ld]; }
    load_idx(wt + NW);
    const int nrow = min(32, count - wt * 32);
    {
      const int perm = hp_ld & 31;
      const int t_id = t_ld | ((hp_ld & 0x40) ? kHeavyBit : 0), h_id = h_ld | ((hp_ld & 0x80) ? kHeavyBit : 0);
      const int h_rank = __shfl(h_id, perm);                    // head of rank r
      const int t_next = __shfl_down(t_id, 1), h_next = __shfl_down(h_rank, 1);
      const bool stop = r + 1 == nrow || (r + 1) % RP == 0;
      const int t_flag = (r < nrow && (stop || t_next != t_id)) ? (int)0x80000000 : 0;
      const int h_flag = (r < nrow && (stop || h_next != h_rank)) ? (int)0x80000000 : 0;
      if (hh == 0) {
        gs_s[r] = g_ld; pi_s[r] = p_ld; hd_s[r] = h_ld; hp_s[r] = perm;
        tl_s[r] = t_id | t_flag; hr_s[r] = h_rank | h_flag;
        st_s[r] = nt.s; sh_s[r] = nh.s;
      }
    }
    // the codes as bfloat16 values (exact): operand fragments of step 1a, and the code matrices
    Bf16Frag tc[NM], hc[NM];
    float mid_t, mid_h;
    {
      // (centred on the row's own mean code, rounded to an integer m: code - m is a small integer,
      // an exact bfloat16 value like the code, and e_hat = mid + scale (code - m) with
      // mid = Z + scale m splits every sum into a part of the size of the row's spread and a part
      // of the size of its mean, instead of two parts of the size of |Z| that cancel)
      const float mt = rintf(code_sum(nt) * (1.0f / (float)D)), mh = rintf(code_sum(nh) * (1.0f / (float)D));
      auto pack = [](uint32_t c0, uint32_t c1, float m) {
        return __builtin_amdgcn_perm(__float_as_uint((float)c1 - m), __float_as_uint((float)c0 - m), 0x07060302u);
      };
      mid_t = fmaf(nt.s, mt, nt.z);
      mid_h = fmaf(nh.s, mh, nh.z);
#pragma unroll
      for (int m = 0; m < NM; ++m) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          tc[m].u[i] = pack(nt.code(8 * m + 2 * i), nt.code(8 * m + 2 * i + 1), mt);
          hc[m].u[i] = pack(nh.code(8 * m + 2 * i), nh.code(8 * m + 2 * i + 1), mh);
        }
        *reinterpret_cast<uint4*>(Ct_s + r * LDW + hh * KH + 8 * m) = *reinterpret_cast<const uint4*>(tc[m].u);
        *reinterpret_cast<uint4*>(Ch_s + r * LDW + hh * KH + 8 * m) = *reinterpret_cast<const uint4*>(hc[m].u);
      }
    }
    if (hh == 0) { zt_s[r] = mid_t; zh_s[r] = mid_h; }
    phase_fence();

    // ---- 1a. code products: accumulator row = edge, lane column = channel
    floatx16 accA[NB], accB[NB];
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) { accA[cb] = floatx16{0}; accB[cb] = floatx16{0}; }
    {
      int wofs = 0;
      asm volatile("" : "+v"(wofs));    // the pieces are re-read from LDS, never parked in registers
      const uint16_t* wrow = Wp + r * LDW + hh * KH + wofs;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        Bf16Frag wh[NB], wm[NB], wl[NB];
#pragma unroll
        for (int cb = 0; cb < NB; ++cb) {
          const uint16_t* wp = wrow + cb * 32 * LDW + 8 * m;
          *reinterpret_cast<uint4*>(wh[cb].u) = *reinterpret_cast<const uint4*>(wp);
          *reinterpret_cast<uint4*>(wm[cb].u) = *reinterpret_cast<const uint4*>(wp + D * LDW);
          *reinterpret_cast<uint4*>(wl[cb].u) = *reinterpret_cast<const uint4*>(wp + 2 * D * LDW);
        }
#define TINYKG_CODE_STEP(WP)                                                                               \
        _Pragma("unroll") for (int cb = 0; cb < NB; ++cb) {                                                \
          accA[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[m].v, WP[cb].v, accA[cb], 0, 0, 0);        \
          accB[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hc[m].v, WP[cb].v, accB[cb], 0, 0, 0);        \
        }
        TINYKG_CODE_STEP(wl)
        TINYKG_CODE_STEP(wm)
        TINYKG_CODE_STEP(wh)
#undef TINYKG_CODE_STEP
        __builtin_amdgcn_sched_barrier(0);   // one k-step's fragments at a time
      }
    }
    // ---- 1b. a = s_t acc + Z_t (W_r 1), b = s_h acc + Z_h (W_r 1) + e_r;
    //          grad_a = gs tanh(b), grad_b = gs a (1 - tanh(b)^2), in place
    float zw_t[NB];          // sum over this lane's edges of mid_t grad_a + mid_h grad_b, channel cb * 32 + r
    {
      float er_t[NB];
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) { er_t[cb] = 0.f; zw_t[cb] = 0.f; }
#pragma unroll
      for (int q = 0; q < 4; ++q) {                    // registers 4q .. 4q + 3: edges 8q + 4hh + u
        const float4 g4 = *reinterpret_cast<const float4*>(gs_s + 8 * q + 4 * hh);
        const float4 a4 = *reinterpret_cast<const float4*>(st_s + 8 * q + 4 * hh);
        const float4 b4 = *reinterpret_cast<const float4*>(sh_s + 8 * q + 4 * hh);
        const float4 c4 = *reinterpret_cast<const float4*>(zt_s + 8 * q + 4 * hh);
        const float4 d4 = *reinterpret_cast<const float4*>(zh_s + 8 * q + 4 * hh);
        const float gq[4] = {g4.x, g4.y, g4.z, g4.w}, stq[4] = {a4.x, a4.y, a4.z, a4.w};
        const float shq[4] = {b4.x, b4.y, b4.z, b4.w}, ztq[4] = {c4.x, c4.y, c4.z, c4.w};
        const float zhq[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
          for (int cb = 0; cb < NB; ++cb) {
            const int v = 4 * q + u;
            const float a = fmaf(stq[u], accA[cb][v], ztq[u] * ws_c[cb]);
            const float b = fmaf(shq[u], accB[cb][v], fmaf(zhq[u], ws_c[cb], er_c[cb]));
            const float vv = tanh_rel(b);
            const float db = gq[u] * a * (1.f - vv * vv);
            const float da = gq[u] * vv;
            accA[cb][v] = da;
            accB[cb][v] = db;
            er_t[cb] += db;
            zw_t[cb] = fmaf(ztq[u], da, fmaf(zhq[u], db, zw_t[cb]));
          }
        }
      }
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) er_acc[cb] += er_t[cb];
    }
    // ---- 1c. grad_W_r[c][i] += sum_e (s_t grad_a)[e][c] code_t[e][i] + (s_h grad_b)[e][c] code_h[e][i]
    //      (a fresh accumulator per tile keeps the fp32 running sum short)
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      floatx16 accT[NB];
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) accT[ib] = floatx16{0};
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int side = 0; side < 2; ++side) {
          // pieces of the scaled gradients of registers 8 ks .. 8 ks + 7 (edges 16 ks + 4 hh + {0..3, 8..11})
          const float* sc_s = side == 0 ? st_s : sh_s;
          const uint16_t* C_s = side == 0 ? Ct_s : Ch_s;
          Bf16Frag xh, xm, xl;
          {
            const float4 s0 = *reinterpret_cast<const float4*>(sc_s + 16 * ks + 4 * hh), s1 = *reinterpret_cast<const float4*>(sc_s + 16 * ks + 8 + 4 * hh);
            const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            float x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = sv[j] * (side == 0 ? accA[cb][8 * ks + j] : accB[cb][8 * ks + j]);
            split3x8(x, xh, xm, xl);
          }
          // codes of column ib * 32 + r at the eight edges of this lane half and k-step
          Bf16Frag cf[NB];
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) {
            const uint2 lo = lds_column4(C_s, LDW, 16 * ks + 4 * hh, ib * 32, lane);
            const uint2 hi = lds_column4(C_s, LDW, 16 * ks + 8 + 4 * hh, ib * 32, lane);
            cf[ib].u[0] = lo.x; cf[ib].u[1] = lo.y; cf[ib].u[2] = hi.x; cf[ib].u[3] = hi.y;
          }
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) accT[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, cf[ib].v, accT[ib], 0, 0, 0);
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) accT[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xm.v, cf[ib].v, accT[ib], 0, 0, 0);
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) accT[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, cf[ib].v, accT[ib], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // the tile's rank-one part (sum_e mid_e grad[e][c]) 1^T joins the tile's sum here, so that the
      // long running sum carries the net value: row c of the block needs the sum of channel c,
      // which lane c % 32 holds (both halves of the wave together)
      {
        const float zc = zw_t[cb] + __shfl_xor(zw_t[cb], 32);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float zr = __shfl(zc, acc_row(v, lane));
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) accT[ib][v] += zr;
        }
      }
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) {
        accW[cb * NB + ib] += accT[ib];
        asm volatile("" : "+v"(accW[cb * NB + ib]));   // pins the addition here
      }
    }
    phase_fence();   // the code matrices are dead from here on: G_s overlays them

    const int si = lane % D, se0 = (lane / D) * RP;   // scatter: this lane's column and rows
    // ---- 2. per side: G_s <- grad (as [e][c]); P = G W_r on the bf16 matrix cores (rows split on
    //      the fly, pieces of W_r^T from LDS); G_s <- P (as [e][i]); rows walked in tail order
    //      resp. head order with running sums, one atomic per run and column
#pragma unroll
    for (int side = 0; side < 2; ++side) {
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          G_s[acc_row(v, lane) * LD + cb * 32 + r] = side == 0 ? accA[cb][v] : accB[cb][v];
      }
      phase_fence();
      floatx16 accP[NB];
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) accP[ib] = floatx16{0};
      {
        int wofs = 0;
        asm volatile("" : "+v"(wofs));
        const uint16_t* wtrow = Wtp + r * LDW + hh * KH + wofs;
        const float* grow = G_s + r * LD + hh * KH;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const float4 lo4 = *reinterpret_cast<const float4*>(grow + 8 * m), hi4 = *reinterpret_cast<const float4*>(grow + 8 * m + 4);
          const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
          Bf16Frag gh, gm, gl;
          split3x8(x, gh, gm, gl);
          Bf16Frag wh[NB], wm[NB], wl[NB];
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) {
            const uint16_t* wp = wtrow + ib * 32 * LDW + 8 * m;
            *reinterpret_cast<uint4*>(wh[ib].u) = *reinterpret_cast<const uint4*>(wp);
            *reinterpret_cast<uint4*>(wm[ib].u) = *reinterpret_cast<const uint4*>(wp + D * LDW);
            *reinterpret_cast<uint4*>(wl[ib].u) = *reinterpret_cast<const uint4*>(wp + 2 * D * LDW);
          }
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) {
            accP[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gh.v, wl[ib].v, accP[ib], 0, 0, 0);
            accP[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gl.v, wh[ib].v, accP[ib], 0, 0, 0);
            accP[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gm.v, wm[ib].v, accP[ib], 0, 0, 0);
            accP[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gh.v, wm[ib].v, accP[ib], 0, 0, 0);
            accP[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gm.v, wh[ib].v, accP[ib], 0, 0, 0);
            accP[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gh.v, wh[ib].v, accP[ib], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // (tails: the e_t term of H_h adds pi_e grad_H_h to the row; the heads' rows of grad_H are fetched
      // in batches of RB rows, each batch requested while the one before it is summed, the first one
      // here, while the products drain)
      constexpr int RB = RP < 8 ? RP : 8;
      float gnext[RB];
      auto fetch_gh = [&](int k0) {
#pragma unroll
        for (int k = 0; k < RB; ++k) {
          const int hk = D == 64 ? __builtin_amdgcn_readfirstlane(hd_s[se0 + k0 + k]) : hd_s[se0 + k0 + k];
          gnext[k] = gH[(int64_t)hk * D + si];
        }
      };
      if (side == 0) fetch_gh(0);
      phase_fence();
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
        for (int v = 0; v < 16; ++v) G_s[acc_row(v, lane) * LD + ib * 32 + r] = accP[ib][v];
      }
      phase_fence();
      float run = 0.f;
#pragma unroll
      for (int k0 = 0; k0 < RP; k0 += RB) {
        int node[RB];
        float val[RB];
        float gcur[RB];
#pragma unroll
        for (int k = 0; k < RB; ++k) gcur[k] = side == 0 ? gnext[k] : 0.f;
        if (side == 0 && k0 + RB < RP) fetch_gh(k0 + RB);
#pragma unroll
        for (int k = 0; k < RB; ++k) {
          if (side == 0) {
            node[k] = tl_s[se0 + k0 + k];
            val[k] = fmaf(pi_s[se0 + k0 + k], gcur[k], G_s[(se0 + k0 + k) * LD + si]);
          } else {
            node[k] = hr_s[se0 + k0 + k];
            const int pk = D == 64 ? __builtin_amdgcn_readfirstlane(hp_s[se0 + k0 + k]) : hp_s[se0 + k0 + k];
            val[k] = G_s[pk * LD + si];
          }
        }
#pragma unroll
        for (int k = 0; k < RB; ++k) {
          run += val[k];
          const int nk = D == 64 ? __builtin_amdgcn_readfirstlane(node[k]) : node[k];
          if (nk < 0) {
            sink_add<D>(sink, nk, si, run);
            run = 0.f;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      phase_fence();   // the other side (or the next tile) overwrites G_s
    }
  }

  // fixed-order combination of the eight waves' partial sums (the buffers overlay everything
  // the span used: every wave must have finished its tiles)
  __syncthreads();
  {
    constexpr int CW = NB * NB * 1024 + D;        // floats per wave
    float* comb = reinterpret_cast<float*>(smem_raw);
    float* mine_c = comb + wave * CW;
#pragma unroll
    for (int j = 0; j < NB * NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) mine_c[(j * 16 + v) * 64 + lane] = accW[j][v];
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      const float both = er_acc[cb] + __shfl_xor(er_acc[cb], 32);
      if (hh == 0) mine_c[NB * NB * 1024 + cb * 32 + r] = both;
    }
    __syncthreads();
    float* outW = part_Wr + (size_t)ch * D * D;
    for (int f = tid; f < D * D; f += NT) {
      const int l = f & 63, v = (f >> 6) & 15, j = f >> 10;
      const int cb = j / NB, ib = j % NB;
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) sum += comb[w * CW + f];
      outW[(cb * 32 + acc_row(v, l)) * D + ib * 32 + (l & 31)] = sum;
    }
    if (tid < D) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) sum += comb[w * CW + NB * NB * 1024 + tid];
      part_er[(size_t)ch * D + tid] = sum;
    }
  }
}

template <int D, int BITS>
__global__ __launch_bounds__(kEdgeWaves * 64) void edge_code_kernel(
    Source src, const float* __restrict__ Wr, const float* __restrict__ er,
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const int32_t* __restrict__ r_eid, const uint8_t* __restrict__ r_hperm, ChunkList spans,
    const int32_t* __restrict__ group_ptr, const float* __restrict__ pi, const float* __restrict__ gs,
    const float* __restrict__ gH, GradSink sink, float* __restrict__ part_Wr, float* __restrict__ part_er) {
  const int first = group_ptr[blockIdx.x], last = group_ptr[blockIdx.x + 1];
  for (int sp = first; sp < last; ++sp) {
    if (sp != first) __syncthreads();   // the previous span's combination has read the waves' partial sums
    edge_code_span<D, BITS>(sp, src, Wr, er, r_head, r_tail, r_eid, r_hperm, spans, pi, gs, gH, sink, part_Wr, part_er);
  }
}

// ----------------------------- edge-level backward, code form, cooperative (d = 128) ----
// The d = 128 edge kernel for a compressed context with one (Z, scale) pair per row, all six
// products on the bf16 matrix cores.  At d = 128 the three bfloat16 pieces of W_r take 102 KiB
// of LDS in ONE layout, so there is no room for W_r^T beside them and none for a region per
// wave: one eight-wave workgroup shares a 32-edge tile (as in the fp32 cooperative kernel
// above, same phases and barriers) and the products that contract over W_r's ROW index read
// W_r column-wise with the transposing LDS read (lds_column4); so do the code columns of 1c.
// The k-loops are unrolled by two, not fully: at 256 registers per wave the fully unrolled
// form makes the register allocator serialise every LDS read with its use (measured 1.7 times slower).
//   stage  rows arrive as raw codes (prefetched a tile ahead); each row's codes are centred on
//          its rounded mean m and stored as bfloat16 (exact): C[e][k] = code - m, with
//          e_hat = mid + scale C, mid = Z + scale m  (Eq. 4)
//   1a     waves 0-3: a, waves 4-7: b for one channel block: three piece products
//          (pieces of W_r) x (codes), then a = s_t acc + mid_t (W_r 1), b likewise + e_r
//   1b     b-waves: grad_a = gs tanh(b) and f = gs (1 - tanh(b)^2) to LDS; a-waves: grad_b = a f
//   1c     every wave two 32 x 32 blocks of grad_W_r += (scale grad)^T C: gradient columns read
//          from LDS, scaled, split three ways in registers; codes read column-wise
//   2      Pt = grad_a W_r (waves 0-3) / Ph = grad_b W_r (waves 4-7), one column block each: rows
//          split on the fly, six piece products against column-wise reads of the pieces of W_r
//   3      Pt, Ph to LDS (over grad_a, grad_b); flag-driven scatter
// The rank-one parts of grad_W_r, (sum_e mid_e grad[e][c]) 1^T, and grad_e_r are column sums
// that every thread keeps for one column and eight of the tile's rows; they join the blocks
// when the chunk is finished.
template <int D>
constexpr int edge_coop_code_smem_bytes() {
  return 3 * D * (D + 16) * 2 + D * 4 + 2 * 32 * (D + 8) * 2 + 2 * 32 * (D + 4) * 4 + 10 * 32 * 4;
}

template <int D, int TE, int BITS>
__global__ __launch_bounds__(kCoopWaves * 64) void edge_coop_code_kernel(
    Source src, const float* __restrict__ Wr, const float* __restrict__ er,
    const int32_t* __restrict__ r_head, const int32_t* __restrict__ r_tail,
    const int32_t* __restrict__ r_eid, const uint8_t* __restrict__ r_hperm, ChunkList chunks,
    const float* __restrict__ pi, const float* __restrict__ gs, const float* __restrict__ gH,
    GradSink sink, float* __restrict__ part_Wr, float* __restrict__ part_er) {
  static_assert(TE == 32 && D == 128 && BITS != 32, "eight waves: four channel blocks x {a, b}; packed rows");
  constexpr int NT = kCoopWaves * 64;
  constexpr int LD = D + 4, LDW = D + 8, LDWW = D + 16, LPR = D / 4, NIB = D / 32;
  constexpr int NBW = NIB * NIB / kCoopWaves;     // grad_W_r blocks per wave (2: one row block, two column blocks)
  constexpr int NQ = NT / D, RP = TE / NQ;        // scatter and column sums: row parts (4 x 8 rows)
  constexpr int CPT = TE * LPR / NT;              // row chunks per thread and matrix (2)
  constexpr int RSTEP = NT / LPR;                 // rows between a thread's chunks
  static_assert(NBW == 2 && NIB % NBW == 0, "a wave's blocks share their row block");
  // (rows of the pieces 288 bytes apart: the four rows of a transposing read then fall into
  // different banks, and so do the 128-bit row reads of eight lanes)
  uint16_t* Wp = reinterpret_cast<uint16_t*>(smem_raw);                 // [3][D][LDWW] pieces of W_r
  float* wsum_s = reinterpret_cast<float*>(Wp + 3 * D * LDWW);          // row sums of W_r
  uint16_t* Ct_s = reinterpret_cast<uint16_t*>(wsum_s + D);             // [TE][LDW] centred codes, tail rows
  uint16_t* Ch_s = Ct_s + TE * LDW;                                     // [TE][LDW] head rows
  float* dA_s = reinterpret_cast<float*>(Ch_s + TE * LDW);              // [TE][LD] grad_a, later Pt
  float* dB_s = dA_s + TE * LD;                                         // [TE][LD] f, grad_b, later Ph
  float* gs_s = dB_s + TE * LD;
  float* pi_s = gs_s + TE;
  float* zt_s = pi_s + TE;                         // (mid, scale) of the tail / head row of edge e
  float* st_s = zt_s + TE;
  float* zh_s = st_s + TE;
  float* sh_s = zh_s + TE;
  int* tl_s = reinterpret_cast<int*>(sh_s + TE);   // tail of row e; sign bit: a tail run ends here
  int* hd_s = tl_s + TE;                           // head of row e
  int* hp_s = hd_s + TE;                           // row of head-order rank k
  int* hr_s = hp_s + TE;                           // head of rank k; sign bit: a head run ends here

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  const int ch = blockIdx.x;
  const int rel = chunks.rel[ch], start = chunks.start[ch], count = chunks.count[ch];
  const int row0 = tid / LPR, li = tid % LPR;     // this thread stages rows row0 + k * RSTEP
  const int blk4 = wave & 3;                      // channel / column block of this wave's products
  const bool b_side = wave >= 4;                  // waves 4-7: b and Ph; waves 0-3: a and Pt

  // prefetch: raw rows of the next tile, node ids of the tile after it
  int tn[CPT], hn[CPT];
  auto load_ids = [&](int t0) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int row = t0 + row0 + k * RSTEP;
      tn[k] = 0; hn[k] = 0;
      if (row < count) { tn[k] = r_tail[start + row]; hn[k] = r_head[start + row]; }
    }
  };
  RawChunk<BITS> rt[CPT], rh[CPT];
  auto load_rows = [&]() {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      rt[k].load(src, (int64_t)tn[k] * LPR + li);
      rh[k].load(src, (int64_t)hn[k] * LPR + li);
    }
  };
  // per-edge scalars of the tile, held by the first wave (lane l and l + 32: row l % 32)
  int t_nx = 0, h_nx = 0, e_nx = -1, hp_nx = 0;
  auto load_edge = [&](int t0) {
    t_nx = 0; h_nx = 0; e_nx = -1; hp_nx = 0;
    if (wave == 0 && t0 + r < count) {
      const int pos = start + t0 + r;
      t_nx = r_tail[pos]; h_nx = r_head[pos]; e_nx = r_eid[pos]; hp_nx = r_hperm[pos];
    }
  };
  float g_ld = 0.f, p_ld = 0.f;
  int t_ld = 0, h_ld = 0, hp_ld = 0;
  auto load_weights = [&]() {
    g_ld = 0.f; p_ld = 0.f;
    if (e_nx >= 0) { g_ld = gs[e_nx]; p_ld = pi[e_nx]; }
    t_ld = t_nx; h_ld = h_nx; hp_ld = hp_nx;
  };
  load_ids(0);
  load_edge(0);
  load_rows();
  load_weights();
  load_ids(TE);
  load_edge(TE);

  stage_split_matrix<D, LDWW>(Wr + (size_t)rel * D * D, Wp, tid, NT);
  for (int c = tid; c < D; c += NT) {
    const float4* row = reinterpret_cast<const float4*>(Wr + ((size_t)rel * D + c) * D);
    double sum = 0.0;
    for (int q = 0; q < D / 4; ++q) { const float4 w = row[q]; sum += (double)w.x + (double)w.y + (double)w.z + (double)w.w; }
    wsum_s[c] = (float)sum;
  }

  floatx16 accW[NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j) accW[j] = floatx16{0};
  const int si = tid % D, se0 = (tid / D) * RP;   // column sums and scatter: this thread's column and rows
  float er_acc = 0.f, zw_acc = 0.f;               // sum_e grad_b[e][si];  sum_e mid_t grad_a + mid_h grad_b

  // four centred codes of a chunk as bfloat16 (exact small integers)
  auto centred = [](uint32_t w, float m) {
    constexpr uint32_t B = (1u << (BITS & 31)) - 1u;
    constexpr int SH = BITS & 31;
    const float c0 = (float)(w & B) - m, c1 = (float)((w >> SH) & B) - m;
    const float c2 = (float)((w >> (2 * SH)) & B) - m, c3 = (float)((w >> (3 * SH)) & B) - m;
    return make_uint2(__builtin_amdgcn_perm(__float_as_uint(c1), __float_as_uint(c0), 0x07060302u),
                      __builtin_amdgcn_perm(__float_as_uint(c3), __float_as_uint(c2), 0x07060302u));
  };
  auto code_sum4 = [](uint32_t w) {
    constexpr uint32_t B = (1u << (BITS & 31)) - 1u;
    constexpr int SH = BITS & 31;
    return (float)((w & B) + ((w >> SH) & B) + ((w >> (2 * SH)) & B) + ((w >> (3 * SH)) & B));
  };

  for (int t0 = 0; t0 < count; t0 += TE) {
    const int nrow = min(TE, count - t0);
    __syncthreads();   // previous tile's scatter has finished reading LDS (first tile: W_r is staged)
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int row = row0 + k * RSTEP;
      // (the 32 lanes of a wave half hold one row: its mean code, rounded to an integer)
      const float mt = rintf(slot_sum<32>(code_sum4(rt[k].w[0])) * (1.0f / (float)D));
      const float mh = rintf(slot_sum<32>(code_sum4(rh[k].w[0])) * (1.0f / (float)D));
      *reinterpret_cast<uint2*>(Ct_s + row * LDW + li * 4) = centred(rt[k].w[0], mt);
      *reinterpret_cast<uint2*>(Ch_s + row * LDW + li * 4) = centred(rh[k].w[0], mh);
      if (li == 0) {
        st_s[row] = rt[k].s; zt_s[row] = fmaf(rt[k].s, mt, rt[k].z);
        sh_s[row] = rh[k].s; zh_s[row] = fmaf(rh[k].s, mh, rh[k].z);
      }
    }
    if (wave == 0) {
      // where the scatter flushes its running sums (see the wave-independent kernel)
      const int perm = hp_ld & 31;
      const int t_id = t_ld | ((hp_ld & 0x40) ? kHeavyBit : 0), h_id = h_ld | ((hp_ld & 0x80) ? kHeavyBit : 0);
      const int h_rank = __shfl(h_id, perm);
      const int t_next = __shfl_down(t_id, 1), h_next = __shfl_down(h_rank, 1);
      const bool stop = r + 1 == nrow || (r + 1) % RP == 0;
      const int t_flag = (r < nrow && (stop || t_next != t_id)) ? (int)0x80000000 : 0;
      const int h_flag = (r < nrow && (stop || h_next != h_rank)) ? (int)0x80000000 : 0;
      if (lane < 32) {
        gs_s[r] = g_ld; pi_s[r] = p_ld; hd_s[r] = h_ld; hp_s[r] = perm;
        tl_s[r] = t_id | t_flag; hr_s[r] = h_rank | h_flag;
      }
    }
    if (t0 + TE < count) {
      load_rows();
      load_weights();
      load_ids(t0 + 2 * TE);
      load_edge(t0 + 2 * TE);
    }
    __syncthreads();
    // ---- 1a. a (waves 0-3) or b (waves 4-7) of channel block blk4 as [c][e], lane = edge:
    //      (pieces of W_r, rows of the block) x (codes), eight k-values per lane half and step
    floatx16 acc1 = {0};
    {
      const uint16_t* wrow = Wp + (blk4 * 32 + r) * LDWW + hh * 8;
      const uint16_t* crow = (b_side ? Ch_s : Ct_s) + r * LDW + hh * 8;
#pragma unroll 2
      for (int m = 0; m < D / 16; ++m) {
        Bf16Frag wh, wm, wl, cf;
        *reinterpret_cast<uint4*>(cf.u) = *reinterpret_cast<const uint4*>(crow + 16 * m);
        *reinterpret_cast<uint4*>(wh.u) = *reinterpret_cast<const uint4*>(wrow + 16 * m);
        *reinterpret_cast<uint4*>(wm.u) = *reinterpret_cast<const uint4*>(wrow + D * LDWW + 16 * m);
        *reinterpret_cast<uint4*>(wl.u) = *reinterpret_cast<const uint4*>(wrow + 2 * D * LDWW + 16 * m);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wl.v, cf.v, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm.v, cf.v, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh.v, cf.v, acc1, 0, 0, 0);
      }
    }
    // ---- 1b. the affine part of Eq. (4), then grad_a and f (b-waves); a stays in registers
    {
      const float sc = b_side ? sh_s[r] : st_s[r], mid = b_side ? zh_s[r] : zt_s[r];
      const float g = gs_s[r];
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int c0 = blk4 * 32 + 8 * vg + 4 * hh;
        const float4 ws4 = *reinterpret_cast<const float4*>(wsum_s + c0);
        const float4 er4 = *reinterpret_cast<const float4*>(er + (size_t)rel * D + c0);   // (cached: 512 bytes per relation)
        const float wsv[4] = {ws4.x, ws4.y, ws4.z, ws4.w}, erv[4] = {er4.x, er4.y, er4.z, er4.w};
        if (b_side) {
          float da[4], f[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float vv = tanh_rel(fmaf(sc, acc1[4 * vg + u], fmaf(mid, wsv[u], erv[u])));
            da[u] = g * vv;
            f[u] = g * (1.f - vv * vv);
          }
          *reinterpret_cast<float4*>(dA_s + r * LD + c0) = make_float4(da[0], da[1], da[2], da[3]);
          *reinterpret_cast<float4*>(dB_s + r * LD + c0) = make_float4(f[0], f[1], f[2], f[3]);
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) acc1[4 * vg + u] = fmaf(sc, acc1[4 * vg + u], mid * wsv[u]);
        }
      }
    }
    __syncthreads();
    // ---- 1b'. grad_b = a * f (the wave that holds a; each element is its own)
    if (!b_side) {
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int c0 = blk4 * 32 + 8 * vg + 4 * hh;
        float4 f = *reinterpret_cast<const float4*>(dB_s + r * LD + c0);
        f.x *= acc1[4 * vg + 0]; f.y *= acc1[4 * vg + 1]; f.z *= acc1[4 * vg + 2]; f.w *= acc1[4 * vg + 3];
        *reinterpret_cast<float4*>(dB_s + r * LD + c0) = f;
      }
    }
    __syncthreads();
    // ---- 1c. grad_W_r blocks [c][i] += sum_e (s_t grad_a)[e][c] C_t[e][i] + (s_h grad_b)[e][c] C_h[e][i]
    //      (a fresh accumulator per tile keeps the fp32 running sum short)
    {
      const int cb = wave / (NIB / NBW), ib0 = (wave % (NIB / NBW)) * NBW;
      floatx16 accT[NBW];
#pragma unroll
      for (int j = 0; j < NBW; ++j) accT[j] = floatx16{0};
#pragma unroll 1
      for (int ks = 0; ks < TE / 16; ++ks) {
#pragma unroll
        for (int side = 0; side < 2; ++side) {
          const float* G_s = side == 0 ? dA_s : dB_s;
          const float* sc_s = side == 0 ? st_s : sh_s;
          const uint16_t* C_s = side == 0 ? Ct_s : Ch_s;
          const int e0 = 16 * ks + 8 * hh;          // this lane half's eight edges of the step
          Bf16Frag xh, xm, xl;
          {
            const float4 s0 = *reinterpret_cast<const float4*>(sc_s + e0), s1 = *reinterpret_cast<const float4*>(sc_s + e0 + 4);
            const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            float x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = sv[i] * G_s[(e0 + i) * LD + cb * 32 + r];
            split3x8(x, xh, xm, xl);
          }
          Bf16Frag cf[NBW];
#pragma unroll
          for (int j = 0; j < NBW; ++j) {
            const uint2 lo = lds_column4(C_s, LDW, e0, (ib0 + j) * 32, lane), hi = lds_column4(C_s, LDW, e0 + 4, (ib0 + j) * 32, lane);
            cf[j].u[0] = lo.x; cf[j].u[1] = lo.y; cf[j].u[2] = hi.x; cf[j].u[3] = hi.y;
          }
#pragma unroll
          for (int j = 0; j < NBW; ++j) accT[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, cf[j].v, accT[j], 0, 0, 0);
#pragma unroll
          for (int j = 0; j < NBW; ++j) accT[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xm.v, cf[j].v, accT[j], 0, 0, 0);
#pragma unroll
          for (int j = 0; j < NBW; ++j) accT[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, cf[j].v, accT[j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int j = 0; j < NBW; ++j) accW[j] += accT[j];
    }
    // grad_H rows of the tile's heads (the e_t term of H_h): requested before the last products
    float ghv[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) ghv[k] = gH[(int64_t)hd_s[se0 + k] * D + si];
    // ---- 2. Pt = grad_a W_r (waves 0-3) or Ph = grad_b W_r (waves 4-7), column block blk4, as [e][i]:
    //      (rows of the gradients, split on the fly) x (pieces of W_r read down its columns)
    floatx16 accP = {0};
    {
      const float* grow = (b_side ? dB_s : dA_s) + r * LD + hh * 8;
#pragma unroll 2
      for (int m = 0; m < D / 16; ++m) {
        const float4 lo4 = *reinterpret_cast<const float4*>(grow + 16 * m), hi4 = *reinterpret_cast<const float4*>(grow + 16 * m + 4);
        const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        Bf16Frag gh, gm, gl, wh, wm, wl;
        split3x8(x, gh, gm, gl);
        {
          const int j0 = 16 * m + 8 * hh;
          const uint2 h0 = lds_column4(Wp, LDWW, j0, blk4 * 32, lane), h1 = lds_column4(Wp, LDWW, j0 + 4, blk4 * 32, lane);
          const uint2 m0 = lds_column4(Wp + D * LDWW, LDWW, j0, blk4 * 32, lane), m1 = lds_column4(Wp + D * LDWW, LDWW, j0 + 4, blk4 * 32, lane);
          const uint2 l0 = lds_column4(Wp + 2 * D * LDWW, LDWW, j0, blk4 * 32, lane), l1 = lds_column4(Wp + 2 * D * LDWW, LDWW, j0 + 4, blk4 * 32, lane);
          wh.u[0] = h0.x; wh.u[1] = h0.y; wh.u[2] = h1.x; wh.u[3] = h1.y;
          wm.u[0] = m0.x; wm.u[1] = m0.y; wm.u[2] = m1.x; wm.u[3] = m1.y;
          wl.u[0] = l0.x; wl.u[1] = l0.y; wl.u[2] = l1.x; wl.u[3] = l1.y;
        }
        mfma_split(gh, gm, gl, wh, wm, wl, accP);
        __builtin_amdgcn_sched_barrier(0);   // one k-step's fragments at a time
      }
    }
    // column sums over this thread's eight rows: grad_e_r and the rank-one part of grad_W_r
    {
      float se = 0.f, sz = 0.f;
#pragma unroll
      for (int k = 0; k < RP; ++k) {
        const float da = dA_s[(se0 + k) * LD + si], db = dB_s[(se0 + k) * LD + si];
        se += db;
        sz = fmaf(zt_s[se0 + k], da, fmaf(zh_s[se0 + k], db, sz));
      }
      er_acc += se;
      zw_acc += sz;
    }
    __syncthreads();   // every read of grad_a / grad_b is done: they become Pt / Ph
    {
      float* P_s = b_side ? dB_s : dA_s;
#pragma unroll
      for (int v = 0; v < 16; ++v) P_s[acc_row(v, lane) * LD + blk4 * 32 + r] = accP[v];
    }
    __syncthreads();
    // scatter: every LDS read is independent of the running sums; a run inside a tile is
    // summed in fp32 and leaves as one atomic per column.  Rows past the end of the chunk
    // carry exact zeros (their weights gs, pi are 0) and no flag.
#pragma unroll
    for (int side = 0; side < 2; ++side) {
      int node[RP];
      float val[RP];
#pragma unroll
      for (int k = 0; k < RP; ++k) {
        if (side == 0) {
          node[k] = tl_s[se0 + k];
          val[k] = fmaf(pi_s[se0 + k], ghv[k], dA_s[(se0 + k) * LD + si]);
        } else {
          node[k] = hr_s[se0 + k];
          val[k] = dB_s[hp_s[se0 + k] * LD + si];
        }
      }
      float run = 0.f;
#pragma unroll
      for (int k = 0; k < RP; ++k) {
        run += val[k];
        if (node[k] < 0) {
          sink_add<D>(sink, node[k], si, run);
          run = 0.f;
        }
      }
    }
  }
  // the four row parts' column sums, in fixed order; the rank-one part joins the blocks
  __syncthreads();
  float* colsum_s = dA_s;                          // [2][NQ][D]
  colsum_s[(tid / D) * D + si] = er_acc;
  colsum_s[(NQ + tid / D) * D + si] = zw_acc;
  __syncthreads();
  float* outW = part_Wr + (size_t)ch * D * D;
  {
    const int cb = wave / (NIB / NBW), ib0 = (wave % (NIB / NBW)) * NBW;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int c = cb * 32 + acc_row(v, lane);
      float zw = 0.f;
#pragma unroll
      for (int q = 0; q < NQ; ++q) zw += colsum_s[(NQ + q) * D + c];
#pragma unroll
      for (int j = 0; j < NBW; ++j) outW[c * D + (ib0 + j) * 32 + r] = accW[j][v] + zw;
    }
  }
  if (tid < D) {
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < NQ; ++q) sum += colsum_s[q * D + tid];
    part_er[(size_t)ch * D + tid] = sum;
  }
}

// The dense backward stage for d_in = d_out = 128 and a compressed H_hat with one (Z, scale)
// pair per row, on the bf16 matrix cores (same outputs as dense_bwd_kernel):
//   grad_H = grad_J W:        (rows of grad_J, split three ways on the fly) x (pieces of W, split once
//                             into LDS, read down their columns with the transposing LDS read): six
//                             piece products
//   grad_W += grad_J^T H_hat: Eq. (4) row by row, H_hat[n] = mid_n + s_n C[n] with C the codes centred on
//                             the row's rounded mean (exact bfloat16 values): (s_n grad_J[n])^T C as three
//                             piece products -- gradient columns read from LDS, scaled, split; code
//                             columns by transposing reads -- plus the rank-one part (sum_n mid_n grad_J[n]) 1^T,
//                             a column sum that each thread keeps for one column and 16 rows of the tile.
// Eight waves: wave w owns block (w & 1, w >> 1) of the 2 x 4 blocks of the grad_H tile and two of
// the sixteen blocks of grad_W (one row block, two column blocks).
constexpr int kDenseCodeWaves = 8;
constexpr int dense_code_smem_bytes() {
  return 3 * 128 * (128 + 16) * 2 + 64 * (128 + 16) * 2 + 64 * (128 + 4) * 4 + 3 * 64 * 4;
}

template <int BITS>
__global__ __launch_bounds__(kDenseCodeWaves * 64) void dense_bwd_code_kernel(
    Source srcH, const uint8_t* __restrict__ mask, const float* __restrict__ gEout, const float* __restrict__ W,
    float slope, int64_t N, float* __restrict__ gH, float* __restrict__ gE, float* __restrict__ part_W,
    double* __restrict__ zero_ptr, int64_t zero_n, const int32_t* __restrict__ deg_rowptr) {
  static_assert(BITS != 32, "packed rows");
  constexpr int D = 128, DO = 128, TN = 64, LD = D + 4, LDW = D + 16, LDWW = DO + 16, LPR = D / 4, NIB = D / 32;
  constexpr int NT = kDenseCodeWaves * 64;
  constexpr int NQ = NT / DO, RP = TN / NQ;       // column sums: row parts (4 x 16 rows)
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < zero_n; i += (int64_t)gridDim.x * NT)
    zero_ptr[i] = 0.0;
  uint16_t* Wp = reinterpret_cast<uint16_t*>(smem_raw);                 // [3][DO][LDWW] pieces of W (rows o)
  uint16_t* C_s = Wp + 3 * DO * LDWW;                                   // [TN][LDW] centred codes of H_hat
  float* gJ_s = reinterpret_cast<float*>(C_s + TN * LDW);               // [TN][LD] grad_J
  float* sc_s = gJ_s + TN * LD;                    // [TN] factor of the grad_H copy in gH (uniform layer: 1 / deg)
  float* s_s = sc_s + TN;                          // [TN] scale of the row
  float* mid_s = s_s + TN;                         // [TN] Z + scale m
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  stage_split_matrix<D, LDWW>(W, Wp, tid, NT);

  floatx16 accW[2];
  accW[0] = floatx16{0}; accW[1] = floatx16{0};
  const int so = tid % DO, sn0 = (tid / DO) * RP;  // column sums: this thread's column and rows
  float zw_acc = 0.f;

  const int64_t n_tiles = (N + TN - 1) / TN;
  constexpr int CPT = TN * LPR / NT, GPT = TN * (DO / 4) / NT;   // 4 and 4
  RawChunk<BITS> preH[CPT];
  float4 preG[GPT];
  uint32_t preM[GPT];
  float preS = 1.f;
  auto load_tile = [&](int64_t tile) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int q = tid + k * NT;
      const int64_t n = tile * TN + q / LPR;
      preH[k].load(srcH, (n < N ? n : 0) * LPR + q % LPR);   // past the end: row 0 (its grad_J row is zero)
    }
    if (deg_rowptr && tid < TN) {
      const int64_t n = tile * TN + tid;
      const int dg = n < N ? deg_rowptr[n + 1] - deg_rowptr[n] : 0;
      preS = dg > 0 ? 1.0f / (float)dg : 0.f;
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int q = tid + k * NT;
      const int64_t n = tile * TN + q / (DO / 4);
      const int c4 = q % (DO / 4);
      preG[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      preM[k] = 0u;
      if (n < N) {
        preG[k] = reinterpret_cast<const float4*>(gEout)[n * (DO / 4) + c4];
        const int64_t bit = (n * (DO / 4) + c4) * 4;
        preM[k] = (mask[bit >> 3] >> (bit & 7)) & 0xFu;
      }
    }
  };
  auto centred = [](uint32_t w, float m) {
    constexpr uint32_t B = (1u << (BITS & 31)) - 1u;
    constexpr int SH = BITS & 31;
    const float c0 = (float)(w & B) - m, c1 = (float)((w >> SH) & B) - m;
    const float c2 = (float)((w >> (2 * SH)) & B) - m, c3 = (float)((w >> (3 * SH)) & B) - m;
    return make_uint2(__builtin_amdgcn_perm(__float_as_uint(c1), __float_as_uint(c0), 0x07060302u),
                      __builtin_amdgcn_perm(__float_as_uint(c3), __float_as_uint(c2), 0x07060302u));
  };
  auto code_sum4 = [](uint32_t w) {
    constexpr uint32_t B = (1u << (BITS & 31)) - 1u;
    constexpr int SH = BITS & 31;
    return (float)((w & B) + ((w >> SH) & B) + ((w >> (2 * SH)) & B) + ((w >> (3 * SH)) & B));
  };
  if (blockIdx.x < n_tiles) load_tile(blockIdx.x);
  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int64_t n0 = tile * TN;
    __syncthreads();   // the previous tile's readers are done (first tile: W is staged)
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int q = tid + k * NT;
      const int row = q / LPR, li = q % LPR;
      // (the 32 lanes of a wave half hold one row: its mean code, rounded to an integer)
      const float m = rintf(slot_sum<32>(code_sum4(preH[k].w[0])) * (1.0f / (float)D));
      *reinterpret_cast<uint2*>(C_s + row * LDW + li * 4) = centred(preH[k].w[0], m);
      if (li == 0) { s_s[row] = preH[k].s; mid_s[row] = fmaf(preH[k].s, m, preH[k].z); }
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int q = tid + k * NT;
      float4 g = preG[k];
      const uint32_t mb = preM[k];
      g.x *= (mb & 1u) ? 1.f : slope; g.y *= (mb & 2u) ? 1.f : slope;
      g.z *= (mb & 4u) ? 1.f : slope; g.w *= (mb & 8u) ? 1.f : slope;
      *reinterpret_cast<float4*>(gJ_s + (q / (DO / 4)) * LD + (q % (DO / 4)) * 4) = g;
    }
    if (tid < TN) sc_s[tid] = preS;
    if (tile + gridDim.x < n_tiles) load_tile(tile + gridDim.x);
    __syncthreads();
    // ---- grad_W blocks [o][i] += sum_n (s_n gJ[n][o]) C[n][i], row block wave / 2, two column blocks
    //      (a fresh accumulator per tile keeps the fp32 running sum short)
    {
      const int ob = wave >> 1, ib0 = (wave & 1) * 2;
      floatx16 accT[2];
      accT[0] = floatx16{0}; accT[1] = floatx16{0};
#pragma unroll 1
      for (int ks = 0; ks < TN / 16; ++ks) {
        const int e0 = 16 * ks + 8 * hh;            // this lane half's eight rows of the step
        Bf16Frag xh, xm, xl;
        {
          const float4 s0 = *reinterpret_cast<const float4*>(s_s + e0), s1 = *reinterpret_cast<const float4*>(s_s + e0 + 4);
          const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
          float x[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = sv[i] * gJ_s[(e0 + i) * LD + ob * 32 + r];
          split3x8(x, xh, xm, xl);
        }
        Bf16Frag cf[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint2 lo = lds_column4(C_s, LDW, e0, (ib0 + j) * 32, lane), hi = lds_column4(C_s, LDW, e0 + 4, (ib0 + j) * 32, lane);
          cf[j].u[0] = lo.x; cf[j].u[1] = lo.y; cf[j].u[2] = hi.x; cf[j].u[3] = hi.y;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) accT[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl.v, cf[j].v, accT[j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 2; ++j) accT[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xm.v, cf[j].v, accT[j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 2; ++j) accT[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh.v, cf[j].v, accT[j], 0, 0, 0);
      }
      accW[0] += accT[0];
      accW[1] += accT[1];
    }
    // ---- grad_H block (nb, ib): [n][i] = sum_o gJ[n][o] W[o][i]
    {
      const int nb = wave & 1, ib = wave >> 1;
      floatx16 acc = {0};
      const float* grow = gJ_s + (nb * 32 + r) * LD + hh * 8;
#pragma unroll 2
      for (int m = 0; m < DO / 16; ++m) {
        const float4 lo4 = *reinterpret_cast<const float4*>(grow + 16 * m), hi4 = *reinterpret_cast<const float4*>(grow + 16 * m + 4);
        const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        Bf16Frag gh, gm, gl, wh, wm, wl;
        split3x8(x, gh, gm, gl);
        {
          const int j0 = 16 * m + 8 * hh;
          const uint2 h0 = lds_column4(Wp, LDWW, j0, ib * 32, lane), h1 = lds_column4(Wp, LDWW, j0 + 4, ib * 32, lane);
          const uint2 m0 = lds_column4(Wp + DO * LDWW, LDWW, j0, ib * 32, lane), m1 = lds_column4(Wp + DO * LDWW, LDWW, j0 + 4, ib * 32, lane);
          const uint2 l0 = lds_column4(Wp + 2 * DO * LDWW, LDWW, j0, ib * 32, lane), l1 = lds_column4(Wp + 2 * DO * LDWW, LDWW, j0 + 4, ib * 32, lane);
          wh.u[0] = h0.x; wh.u[1] = h0.y; wh.u[2] = h1.x; wh.u[3] = h1.y;
          wm.u[0] = m0.x; wm.u[1] = m0.y; wm.u[2] = m1.x; wm.u[3] = m1.y;
          wl.u[0] = l0.x; wl.u[1] = l0.y; wl.u[2] = l1.x; wl.u[3] = l1.y;
        }
        mfma_split(gh, gm, gl, wh, wm, wl, acc);
        __builtin_amdgcn_sched_barrier(0);   // one k-step's fragments at a time
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t n = n0 + nb * 32 + acc_row(v, lane);
        if (n < N) {
          gH[n * D + ib * 32 + r] = acc[v] * sc_s[nb * 32 + acc_row(v, lane)];
          gE[n * D + ib * 32 + r] = acc[v];
        }
      }
    }
    // column sums over this thread's sixteen rows: the rank-one part of grad_W
    {
      float sz = 0.f;
#pragma unroll
      for (int k = 0; k < RP; ++k) sz = fmaf(mid_s[sn0 + k], gJ_s[(sn0 + k) * LD + so], sz);
      zw_acc += sz;
    }
  }
  // the row parts' column sums, in fixed order; the rank-one part joins the blocks
  __syncthreads();
  float* colsum_s = gJ_s;                          // [NQ][DO]
  colsum_s[(tid / DO) * DO + so] = zw_acc;
  __syncthreads();
  float* out = part_W + (size_t)blockIdx.x * DO * D;
  {
    const int ob = wave >> 1, ib0 = (wave & 1) * 2;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int o = ob * 32 + acc_row(v, lane);
      float zw = 0.f;
#pragma unroll
      for (int q = 0; q < NQ; ++q) zw += colsum_s[q * DO + o];
#pragma unroll
      for (int j = 0; j < 2; ++j) out[o * D + (ib0 + j) * 32 + r] = accW[j][v] + zw;
    }
  }
}

// ------------------------------------------------------------- host helpers ----
size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

bool dims_ok(int d_in, int d_rel, int d_out) {
  return d_in == d_rel && (d_in == 32 || d_in == 64 || d_in == 128) && d_out >= 16 && d_out <= 128 &&
         d_out % 16 == 0;
}

int dense_grid(int64_t N) {
  const int64_t tiles = (N + 63) / 64;
  const int64_t cap = (int64_t)num_cus() * 2;
  return (int)std::max<int64_t>(1, std::min(tiles, cap));
}

struct HeavyWs { size_t pm, pz, pacc, pc, hm, hz, end; };
HeavyWs heavy_layout(const tinykg_graph* g, int d, size_t at) {
  HeavyWs w;
  w.pm = at;
  w.pz = w.pm + align256((size_t)g->n_hseg * 4);
  w.pacc = w.pz + align256((size_t)g->n_hseg * 8);
  w.pc = w.pacc + align256((size_t)g->n_hseg * d * 8);
  w.hm = w.pc + align256((size_t)g->n_hseg * 8);
  w.hz = w.hm + align256((size_t)g->n_heavy * 4);
  w.end = w.hz + align256((size_t)g->n_heavy * 8);
  return w;
}

HeavyList heavy_list(const tinykg_graph* g) {
  return HeavyList{g->heavy_head, g->heavy_seg_ptr, g->hseg_q, g->hseg_e0, g->hseg_cnt, g->n_heavy,
                   g->n_hseg};
}

struct FwdWs { size_t s, H, total; HeavyWs hv; };
FwdWs fwd_layout(const tinykg_graph* g, int d) {
  FwdWs w;
  w.s = 0;
  w.H = align256((size_t)g->n_edges * 4);
  w.hv = heavy_layout(g, d, w.H + align256((size_t)g->n_nodes * d * 4));
  w.total = w.hv.end;
  return w;
}

struct BwdWs { size_t s, pi, gs, gH, acc, pW, pWr, per, total; HeavyWs hv; };
BwdWs bwd_layout(const tinykg_graph* g, int d, int d_out) {
  BwdWs w;
  const size_t e = align256((size_t)g->n_edges * 4);
  w.s = 0; w.pi = e; w.gs = 2 * e; w.gH = 3 * e;
  w.acc = w.gH + align256((size_t)g->n_nodes * d * 4);
  w.pW = w.acc + align256((size_t)g->n_acc_heavy * kHeavyReplicas * d * 8);
  w.pWr = w.pW + align256((size_t)dense_grid(g->n_nodes) * d_out * d * 4);
  // (one partial per chunk, or per span of the persistent kernel, whichever are more)
  const size_t n_part = (size_t)std::max(g->n_chunks, std::max(g->n_spans, g->n_espans));
  w.per = w.pWr + align256(n_part * d * d * 4);
  w.hv = heavy_layout(g, d, w.per + align256(n_part * d * 4));
  w.total = w.hv.end;
  return w;
}

template <typename Kern>
tinykg_status set_smem(Kern k, size_t bytes) {
  if (bytes > 160 * 1024) return TINYKG_ERR_UNSUPPORTED;
  if (bytes > 48 * 1024)
    TINYKG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return TINYKG_OK;
}

template <int D, int BITS>
tinykg_status launch_score(const tinykg_graph* g, Source src, const float* Wr, const float* er,
                           float* s, hipStream_t st) {
  if (g->n_chunks == 0) return TINYKG_OK;
  ChunkList cl{g->chunk_rel, g->chunk_start, g->chunk_count};
  ProfileScope prof("score_kernel", st);
  if constexpr (D <= 64) {
    const size_t smem = (size_t)3 * D * (D + 8) * 2 + (size_t)2 * D * 4;
    auto kern = score_split_kernel<D, BITS, false>;
    if constexpr (BITS != 32) {
      if ((4 << src.group_chunks_log2) >= D) kern = score_split_kernel<D, BITS, true>;   // one group per row
    }
    tinykg_status rc = set_smem(kern, smem);
    if (rc != TINYKG_OK) return rc;
    hipLaunchKernelGGL(kern, dim3(g->n_chunks), dim3(kScoreWaves * 64), smem, st, src, Wr, er, g->r_head,
                       g->r_tail, g->r_eid, cl, s);
  } else {
    constexpr int TE = 32;
    // (tile: three bfloat16 pieces per side, or one matrix of codes per side)
    size_t smem = (size_t)3 * 2 * TE * (D + 8) * 2 + (size_t)(2 * D + (D / 32) * 2 * TE + 4 * TE) * 4;
    auto kern = score_coop_split_kernel<D, TE, BITS, false>;
    if constexpr (BITS != 32) {
      if ((4 << src.group_chunks_log2) >= D) {
        kern = score_coop_split_kernel<D, TE, BITS, true>;
        smem = (size_t)2 * TE * (D + 8) * 2 + (size_t)(2 * D + (D / 32) * 2 * TE + 4 * TE) * 4;
      }
    }
    tinykg_status rc = set_smem(kern, smem);
    if (rc != TINYKG_OK) return rc;
    hipLaunchKernelGGL(kern, dim3(g->n_chunks), dim3(kThreads), smem, st, src, Wr, er, g->r_head,
                       g->r_tail, g->r_eid, cl, s);
  }
  return launch_status();
}

// H_h = e_h + sum_j pi_j e_t from the rows behind `src` (exact E in the forward pass; the
// saved E_hat when the backward pass rebuilds H instead of reading a saved copy).
template <int D, int BITS>
tinykg_status launch_attend_fwd(const tinykg_graph* g, Source src, const float* s, float* H, uint8_t* ws,
                                const HeavyWs& hv, hipStream_t st) {
  const int64_t N = g->n_nodes;
  tinykg_status rc;
  const int wave_blocks = (int)std::max<int64_t>(1, std::min<int64_t>((N + 3) / 4, (int64_t)num_cus() * 16));
  {
    ProfileScope prof("attend_fwd_kernel", st);
    hipLaunchKernelGGL((attend_fwd_kernel<D, BITS>), dim3(wave_blocks), dim3(kThreads), 0, st, src, g->rowptr,
                       g->h_tail, s, N, H);
  }
  if ((rc = launch_status()) != TINYKG_OK) return rc;
  if (g->n_heavy > 0) {
    const HeavyList hl = heavy_list(g);
    float* pm = reinterpret_cast<float*>(ws + hv.pm);
    double* pz = reinterpret_cast<double*>(ws + hv.pz);
    double* pacc = reinterpret_cast<double*>(ws + hv.pacc);
    float* hm = reinterpret_cast<float*>(ws + hv.hm);
    double* hz = reinterpret_cast<double*>(ws + hv.hz);
    ProfileScope prof("heavy_head_kernels", st);
    hipLaunchKernelGGL((heavy_part1_kernel<D, true, BITS>), dim3((g->n_hseg + 3) / 4), dim3(kThreads), 0, st,
                       src, g->h_tail, s, hl, pm, pz, pacc);
    hipLaunchKernelGGL((heavy_merge1_kernel<D, true, BITS>), dim3(g->n_heavy), dim3(kMergeWaves * 64), 0, st,
                       src, hl, pm, pz, pacc, hm, hz, H);
    if ((rc = launch_status()) != TINYKG_OK) return rc;
  }
  return TINYKG_OK;
}

template <int D>
tinykg_status fwd_impl(const tinykg_graph* g, const float* E, const float* Wr, const float* er,
                       const float* W, int d_out, float slope, int bits, int group, uint64_t seed,
                       float* E_out, const tinykg_saved* sv, uint8_t* ws, hipStream_t st, bool uniform) {
  const int64_t N = g->n_nodes;
  const FwdWs L = fwd_layout(g, D);
  float* s = reinterpret_cast<float*>(ws + L.s);
  const bool keep_H = sv->packed_H != nullptr;   // else: the backward pass rebuilds H from E_hat
  float* H = bits == 32 && keep_H ? reinterpret_cast<float*>(sv->packed_H) : reinterpret_cast<float*>(ws + L.H);
  Source src{reinterpret_cast<const uint8_t*>(E), nullptr, nullptr, 0};
  tinykg_status rc = TINYKG_OK;
  if (uniform) {                          // pi = 1 / deg: the softmax of all-zero scores
    if (g->n_edges > 0) {
      ProfileScope prof("zero_scores_kernel", st);
      const int blocks = (int)std::min<int64_t>((g->n_edges + 255) / 256, (int64_t)num_cus() * 16);
      hipLaunchKernelGGL(zero_f32_fill_kernel, dim3(blocks), dim3(256), 0, st, s, g->n_edges);
      rc = launch_status();
    }
  } else {
    rc = launch_score<D, 32>(g, src, Wr, er, s, st);
  }
  if (rc != TINYKG_OK) return rc;
  if ((rc = launch_attend_fwd<D, 32>(g, src, s, H, ws, L.hv, st)) != TINYKG_OK) return rc;
  // save the context (Fig. 1): Q(E; seed), Q(H; seed + 1)
  // (the uniform layer's backward pass never reads E: only Q(H) and the mask are kept)
  if (bits == 32) {
    if (!uniform) {
      ProfileScope prof("copy_E_fp32", st);
      TINYKG_HIP_TRY(hipMemcpyAsync(sv->packed_E, E, (size_t)N * D * 4, hipMemcpyDeviceToDevice, st));
    }
  } else {
    if (!uniform) {
      rc = launch_quantize(E, N * D, bits, group, seed, 0, TINYKG_ROUND_STOCHASTIC, sv->packed_E,
                           sv->gmin_E, sv->gscale_E, st);
      if (rc != TINYKG_OK) return rc;
    }
    if (keep_H) {
      rc = launch_quantize(H, N * D, bits, group, seed + 1, 0, TINYKG_ROUND_STOCHASTIC, sv->packed_H,
                           sv->gmin_H, sv->gscale_H, st);
      if (rc != TINYKG_OK) return rc;
    }
  }
  const int DOP = (d_out + 31) & ~31;
  const size_t smem = (size_t)(64 * (D + 4) + 64 * (DOP + 4)) * 4;
  auto kern = dense_fwd_kernel<D>;
  if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
  ProfileScope prof("dense_fwd_kernel", st);
  // (persistent workgroups, as many as stay resident: LDS allows two at d = 128, four below)
  const int fwd_grid = (int)std::max<int64_t>(1, std::min<int64_t>((N + 63) / 64, (int64_t)num_cus() * (D == 128 ? 2 : 4)));
  hipLaunchKernelGGL(kern, dim3(fwd_grid), dim3(kThreads), smem, st, H, W, d_out, slope, N,
                     E_out, sv->mask_J);
  return launch_status();
}

template <int D, int BITS>
tinykg_status bwd_impl(const tinykg_graph* g, const tinykg_saved* sv, const float* Wr,
                       const float* er, const float* W, int d_out, float slope, int group,
                       const float* gEout, float* gE, float* gWr, float* ger, float* gW,
                       uint8_t* ws, hipStream_t st, bool uniform) {
  constexpr int TE = 32;   // edge tile of the d = 128 kernel
  constexpr int LD = D + 4;
  const int64_t N = g->n_nodes;
  const BwdWs L = bwd_layout(g, D, d_out);
  float* s = reinterpret_cast<float*>(ws + L.s);
  float* pi = reinterpret_cast<float*>(ws + L.pi);
  float* gs = reinterpret_cast<float*>(ws + L.gs);
  float* gH = reinterpret_cast<float*>(ws + L.gH);
  double* acc = reinterpret_cast<double*>(ws + L.acc);
  float* pW = reinterpret_cast<float*>(ws + L.pW);
  float* pWr = reinterpret_cast<float*>(ws + L.pWr);
  float* per = reinterpret_cast<float*>(ws + L.per);
  const int gl2 = BITS == 32 ? 0 : ilog2(group / 4);
  Source srcE{sv->packed_E, sv->gmin_E, sv->gscale_E, gl2};
  Source srcH{sv->packed_H, sv->gmin_H, sv->gscale_H, gl2};
  tinykg_status rc = TINYKG_OK;
  // which partial sums of grad_W_r / grad_e_r belong to relation r (per span of the persistent
  // kernel that ran, per chunk from the d = 128 one)
  const int32_t* part_ptr = D <= 64 ? g->rel_span_ptr : g->rel_chunk_ptr;

  // (uniform: pi = 1 / deg, only the transposed sparse product is left)
  // H was not saved: rebuild it from E_hat (scores first), in the buffer that grad_H then
  // overwrites tile by tile (the dense kernel reads the rows of a tile before it writes them)
  const bool rebuild_H = sv->packed_H == nullptr;
  bool have_scores = false;
  if (rebuild_H) {
    if (g->n_chunks > 0) {
      if ((rc = launch_score<D, BITS>(g, srcE, Wr, er, s, st)) != TINYKG_OK) return rc;
      have_scores = true;
    }
    if ((rc = launch_attend_fwd<D, BITS>(g, srcE, s, gH, ws, L.hv, st)) != TINYKG_OK) return rc;
    srcH = Source{reinterpret_cast<const uint8_t*>(gH), nullptr, nullptr, 0};
  }
  // dense stage
  const int DOP = (d_out + 31) & ~31;
  const int64_t n_heavy_elems = (int64_t)g->n_acc_heavy * D;
  const bool with_heavy = g->n_edges > 0 && n_heavy_elems > 0;
  int dense_blocks = 0;
  {
    const int grid = dense_grid(N);
    dense_blocks = grid;
    bool code_form = false;
    if constexpr (D == 128 && BITS != 32) {
      // (d_in = d_out = 128, H_hat saved with one (Z, scale) pair per row: everything on the bf16 matrix cores)
      code_form = !rebuild_H && d_out == 128 && group >= D;
      if (code_form) {
        const size_t smem = (size_t)dense_code_smem_bytes();
        auto kern = dense_bwd_code_kernel<BITS>;
        if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
        ProfileScope prof("dense_bwd_kernel", st);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kDenseCodeWaves * 64), smem, st, srcH, sv->mask_J, gEout, W,
                           slope, N, gH, gE, pW, acc, with_heavy ? n_heavy_elems * kHeavyReplicas : 0,
                           uniform ? g->rowptr : (const int32_t*)nullptr);
      }
    }
    if (!code_form) {
      const size_t smem = (size_t)(DOP * LD + 64 * LD + 64 * (DOP + 4) + 64) * 4;
      auto kern = rebuild_H ? dense_bwd_kernel<D, 32> : dense_bwd_kernel<D, BITS>;
      if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
      ProfileScope prof("dense_bwd_kernel", st);
      hipLaunchKernelGGL(kern, dim3(grid), dim3(dense_bwd_waves<D>() * 64), smem, st, srcH, sv->mask_J, gEout, W,
                         d_out, slope, N, gH, gE, pW, acc, with_heavy ? n_heavy_elems * kHeavyReplicas : 0,
                         uniform ? g->rowptr : (const int32_t*)nullptr);
    }
    if ((rc = launch_status()) != TINYKG_OK) return rc;
  }
  if (uniform && g->n_edges > 0) {
    const GradSink sink{gE, acc, g->acc_slot};
    const int64_t waves = (g->n_edges + 31) / 32;
    ProfileScope prof("uniform_bwd_kernel", st);
    hipLaunchKernelGGL((uniform_tail_kernel<D>), dim3((unsigned)((waves + 3) / 4)), dim3(kThreads), 0, st,
                       g->c_head, g->c_tail, gH, g->n_edges, sink);
    if ((rc = launch_status()) != TINYKG_OK) return rc;
  }
  if (!uniform && g->n_chunks > 0) {
    if (!have_scores && (rc = launch_score<D, BITS>(g, srcE, Wr, er, s, st)) != TINYKG_OK) return rc;
    const int wave_blocks = (int)std::max<int64_t>(1, std::min<int64_t>((N + 3) / 4, (int64_t)num_cus() * 16));
    {
      ProfileScope prof("attend_bwd_kernel", st);
      hipLaunchKernelGGL((attend_bwd_kernel<D, BITS>), dim3(wave_blocks), dim3(kThreads), 0, st, srcE,
                         gH, g->rowptr, g->h_tail, s, N, pi, gs);
    }
    if ((rc = launch_status()) != TINYKG_OK) return rc;
    if (g->n_heavy > 0) {
      const HeavyList hl = heavy_list(g);
      float* pm = reinterpret_cast<float*>(ws + L.hv.pm);
      double* pz = reinterpret_cast<double*>(ws + L.hv.pz);
      double* pc = reinterpret_cast<double*>(ws + L.hv.pc);
      float* hm = reinterpret_cast<float*>(ws + L.hv.hm);
      double* hz = reinterpret_cast<double*>(ws + L.hv.hz);
      ProfileScope prof("heavy_head_kernels", st);
      const dim3 gs_grid((g->n_hseg + 3) / 4), gh_grid(g->n_heavy);
      if (!rebuild_H) {   // else the rebuild of H left the softmax statistics of the heavy heads in hm / hz
        hipLaunchKernelGGL((heavy_part1_kernel<D, false, BITS>), gs_grid, dim3(kThreads), 0, st,
                           srcE, g->h_tail, s, hl, pm, pz, (double*)nullptr);
        hipLaunchKernelGGL((heavy_merge1_kernel<D, false, BITS>), gh_grid, dim3(kMergeWaves * 64), 0, st,
                           srcE, hl, pm, pz, (const double*)nullptr, hm, hz, (float*)nullptr);
      }
      hipLaunchKernelGGL((heavy_part2_kernel<D, BITS>), gs_grid, dim3(kThreads), 0, st, srcE, gH, g->h_tail,
                         s, hl, hm, hz, pi, gs, pc);
      hipLaunchKernelGGL(heavy_part3_kernel, gs_grid, dim3(kThreads), 0, st, hl, pc, pi, gs);
      if ((rc = launch_status()) != TINYKG_OK) return rc;
    }
    ChunkList cl{g->chunk_rel, g->chunk_start, g->chunk_count};
    const GradSink sink{gE, acc, g->acc_slot};
    if constexpr (D <= 64) {
      bool code_form = false;
      if constexpr (BITS != 32) code_form = group >= D;   // one (Z, scale) pair per row
      part_ptr = code_form ? g->rel_espan_ptr : g->rel_span_ptr;
      if constexpr (BITS != 32) {
        if (code_form) {
          const size_t smem = (size_t)edge_code_smem_bytes<D>();
          auto kern = edge_code_kernel<D, BITS>;
          if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
          ProfileScope prof("edge_bwd_kernel", st);
          const ChunkList spans{g->espan_rel, g->espan_start, g->espan_count};
          hipLaunchKernelGGL(kern, dim3(g->n_span_groups), dim3(kEdgeWaves * 64), smem, st, srcE, Wr, er,
                             g->r_head, g->r_tail, g->r_eid, g->r_hperm32, spans, g->espan_group_ptr, pi, gs, gH,
                             sink, pWr, per);
        }
      }
      if (!code_form) {
        const size_t smem = (size_t)(D * LD + D + kEdgeWaves * edge_wave_region<D>()) * 4;
        auto kern = edge_wave_kernel<D, BITS>;
        if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
        ProfileScope prof("edge_bwd_kernel", st);
        const ChunkList spans{g->span_rel, g->span_start, g->span_count};
        hipLaunchKernelGGL(kern, dim3(g->n_span_groups), dim3(kEdgeWaves * 64), smem, st, srcE, Wr, er,
                           g->r_head, g->r_tail, g->r_eid, g->r_hperm32, spans, g->span_group_ptr, pi, gs, gH,
                           sink, pWr, per);
      }
    } else {
      bool code_form = false;
      if constexpr (BITS != 32) code_form = group >= D;   // one (Z, scale) pair per row
      if constexpr (BITS != 32) {
        if (code_form) {
          const size_t smem = (size_t)edge_coop_code_smem_bytes<D>();
          auto kern = edge_coop_code_kernel<D, TE, BITS>;
          if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
          ProfileScope prof("edge_bwd_kernel", st);
          hipLaunchKernelGGL(kern, dim3(g->n_chunks), dim3(kCoopWaves * 64), smem, st, srcE, Wr, er, g->r_head,
                             g->r_tail, g->r_eid, g->r_hperm32, cl, pi, gs, gH, sink, pWr, per);
        }
      }
      if (!code_form) {
        const size_t smem = (size_t)(D * LD + 4 * TE * LD + D + 6 * TE + 2 * D + 4) * 4;
        auto kern = edge_bwd_kernel<D, TE, BITS>;
        if ((rc = set_smem(kern, smem)) != TINYKG_OK) return rc;
        ProfileScope prof("edge_bwd_kernel", st);
        hipLaunchKernelGGL(kern, dim3(g->n_chunks), dim3(kCoopWaves * 64), smem, st, srcE, Wr, er, g->r_head,
                           g->r_tail, g->r_eid, g->r_hperm32, cl, pi, gs, gH, sink, pWr, per);
      }
    }
    if ((rc = launch_status()) != TINYKG_OK) return rc;
  }
  // one launch: grad_W, grad_W_r, grad_e_r from their partial sums; heavy-node rows of grad_E
  {
    const bool edge_grads = !uniform && g->n_rel > 0;
    const ReduceJob jW{pW, nullptr, dense_blocks, d_out * D, (d_out * D + 63) / 64, 1, gW};
    // (partial sums per span from the persistent kernel, per chunk from the d = 128 one)
    // (part_ptr: set where the edge kernel was chosen)
    const ReduceJob jWr{pWr, part_ptr, 0, D * D, edge_grads ? (D * D + 63) / 64 : 0, g->n_rel, gWr};
    const ReduceJob jer{per, part_ptr, 0, D, edge_grads ? (D + 63) / 64 : 0, g->n_rel, ger};
    const HeavyFinish hf{acc, g->acc_node, with_heavy ? n_heavy_elems : 0, D, gE};
    const int gx = std::max(std::max(jW.nx, jWr.nx), std::max(jer.nx, with_heavy ? 64 : 1));
    const int gy = std::max(1, edge_grads ? (int)g->n_rel : 1);
    ProfileScope prof("epilogue_kernel", st);
    hipLaunchKernelGGL(epilogue_kernel, dim3(gx, gy, 4), dim3(256), 0, st, jW, jWr, jer, hf);
    if ((rc = launch_status()) != TINYKG_OK) return rc;
  }
  return TINYKG_OK;
}

template <int D>
tinykg_status bwd_bits(int bits, const tinykg_graph* g, const tinykg_saved* sv, const float* Wr,
                       const float* er, const float* W, int d_out, float slope, int group,
                       const float* gEout, float* gE, float* gWr, float* ger, float* gW,
                       uint8_t* ws, hipStream_t st, bool uniform) {
  switch (bits) {
    case 1: return bwd_impl<D, 1>(g, sv, Wr, er, W, d_out, slope, group, gEout, gE, gWr, ger, gW, ws, st, uniform);
    case 2: return bwd_impl<D, 2>(g, sv, Wr, er, W, d_out, slope, group, gEout, gE, gWr, ger, gW, ws, st, uniform);
    case 4: return bwd_impl<D, 4>(g, sv, Wr, er, W, d_out, slope, group, gEout, gE, gWr, ger, gW, ws, st, uniform);
    case 8: return bwd_impl<D, 8>(g, sv, Wr, er, W, d_out, slope, group, gEout, gE, gWr, ger, gW, ws, st, uniform);
    case 32: return bwd_impl<D, 32>(g, sv, Wr, er, W, d_out, slope, group, gEout, gE, gWr, ger, gW, ws, st, uniform);
  }
  return TINYKG_ERR_INVALID_ARG;
}

// packed_H == NULL: H is not saved (the backward pass rebuilds it from E_hat)
tinykg_status check_saved(const tinykg_saved* sv, int bits) {
  if (!sv || !sv->packed_E || !sv->mask_J) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(sv->packed_E) || !aligned16(sv->packed_H) || !aligned16(sv->mask_J))
    return TINYKG_ERR_INVALID_ARG;
  if (bits != 32) {
    if (!sv->gmin_E || !sv->gscale_E) return TINYKG_ERR_INVALID_ARG;
    if (!aligned16(sv->gmin_E) || !aligned16(sv->gscale_E)) return TINYKG_ERR_INVALID_ARG;
    if (sv->packed_H) {
      if (!sv->gmin_H || !sv->gscale_H) return TINYKG_ERR_INVALID_ARG;
      if (!aligned16(sv->gmin_H) || !aligned16(sv->gscale_H)) return TINYKG_ERR_INVALID_ARG;
    }
  }
  return TINYKG_OK;
}

// the uniform layer keeps only Q(H) and the mask
tinykg_status check_saved_uniform(const tinykg_saved* sv, int bits) {
  if (!sv || !sv->packed_H || !sv->mask_J) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(sv->packed_H) || !aligned16(sv->mask_J)) return TINYKG_ERR_INVALID_ARG;
  if (bits != 32) {
    if (!sv->gmin_H || !sv->gscale_H) return TINYKG_ERR_INVALID_ARG;
    if (!aligned16(sv->gmin_H) || !aligned16(sv->gscale_H)) return TINYKG_ERR_INVALID_ARG;
  }
  return TINYKG_OK;
}

tinykg_status check_common(const tinykg_graph* g, int d_in, int d_rel, int d_out, int bits, int group) {
  if (!g) return TINYKG_ERR_INVALID_ARG;
  if (!(bits == 32 || bits_ok(bits))) return TINYKG_ERR_INVALID_ARG;
  if (bits != 32 && !group_ok(group)) return TINYKG_ERR_INVALID_ARG;
  if (!dims_ok(d_in, d_rel, d_out)) return TINYKG_ERR_UNSUPPORTED;
  if (bits != 32 && (g->n_nodes * d_in) % group != 0) return TINYKG_ERR_SHAPE;
  return TINYKG_OK;
}

}  // namespace

}  // namespace tinykg

extern "C" {

size_t tinykg_kg_aggregate_workspace_bytes(const tinykg_graph* g, int d_in, int d_rel, int d_out,
                                           int is_bwd) {
  using namespace tinykg;
  if (!g || !dims_ok(d_in, d_rel, d_out)) return 0;
  return is_bwd ? bwd_layout(g, d_in, d_out).total : fwd_layout(g, d_in).total;
}

tinykg_status tinykg_kg_aggregate_fwd(const tinykg_graph* g, const float* E, const float* Wr,
                                      const float* er, const float* W, int d_in, int d_rel,
                                      int d_out, float leaky_slope, int bits, int group,
                                      uint64_t seed, float* E_out, const tinykg_saved* saved,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  using namespace tinykg;
  tinykg_status rc = check_common(g, d_in, d_rel, d_out, bits, group);
  if (rc != TINYKG_OK) return rc;
  if ((rc = check_saved(saved, bits)) != TINYKG_OK) return rc;
  if (g->n_nodes == 0) return TINYKG_OK;
  if (!E || !W || !E_out || (g->n_edges > 0 && (!Wr || !er))) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(E) || !aligned16(W) || !aligned16(E_out) || !aligned16(Wr) || !aligned16(er))
    return TINYKG_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace) || workspace_bytes < fwd_layout(g, d_in).total)
    return TINYKG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  switch (d_in) {
    case 32: return fwd_impl<32>(g, E, Wr, er, W, d_out, leaky_slope, bits, group, seed, E_out, saved, ws, st, false);
    case 64: return fwd_impl<64>(g, E, Wr, er, W, d_out, leaky_slope, bits, group, seed, E_out, saved, ws, st, false);
    case 128: return fwd_impl<128>(g, E, Wr, er, W, d_out, leaky_slope, bits, group, seed, E_out, saved, ws, st, false);
  }
  return TINYKG_ERR_UNSUPPORTED;
}

tinykg_status tinykg_kg_aggregate_bwd(const tinykg_graph* g, const tinykg_saved* saved,
                                      const float* Wr, const float* er, const float* W, int d_in,
                                      int d_rel, int d_out, float leaky_slope, int bits, int group,
                                      const float* grad_E_out, float* grad_E, float* grad_Wr,
                                      float* grad_er, float* grad_W, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  using namespace tinykg;
  tinykg_status rc = check_common(g, d_in, d_rel, d_out, bits, group);
  if (rc != TINYKG_OK) return rc;
  if ((rc = check_saved(saved, bits)) != TINYKG_OK) return rc;
  if (!W || !grad_W || !aligned16(W) || !aligned16(grad_W)) return TINYKG_ERR_INVALID_ARG;
  if (g->n_rel > 0 && (!Wr || !er || !grad_Wr || !grad_er)) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(Wr) || !aligned16(er) || !aligned16(grad_Wr) || !aligned16(grad_er))
    return TINYKG_ERR_INVALID_ARG;
  if (g->n_nodes > 0 && (!grad_E_out || !grad_E || !aligned16(grad_E_out) || !aligned16(grad_E)))
    return TINYKG_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace) || workspace_bytes < bwd_layout(g, d_in, d_out).total)
    return TINYKG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  switch (d_in) {
    case 32: return bwd_bits<32>(bits, g, saved, Wr, er, W, d_out, leaky_slope, group, grad_E_out, grad_E, grad_Wr, grad_er, grad_W, ws, st, false);
    case 64: return bwd_bits<64>(bits, g, saved, Wr, er, W, d_out, leaky_slope, group, grad_E_out, grad_E, grad_Wr, grad_er, grad_W, ws, st, false);
    case 128: return bwd_bits<128>(bits, g, saved, Wr, er, W, d_out, leaky_slope, group, grad_E_out, grad_E, grad_Wr, grad_er, grad_W, ws, st, false);
  }
  return TINYKG_ERR_UNSUPPORTED;
}

tinykg_status tinykg_kg_uniform_fwd(const tinykg_graph* g, const float* E, const float* W, int d_in,
                                    int d_out, float leaky_slope, int bits, int group, uint64_t seed,
                                    float* E_out, const tinykg_saved* saved, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  using namespace tinykg;
  tinykg_status rc = check_common(g, d_in, d_in, d_out, bits, group);
  if (rc != TINYKG_OK) return rc;
  if ((rc = check_saved_uniform(saved, bits)) != TINYKG_OK) return rc;
  if (g->n_nodes == 0) return TINYKG_OK;
  if (!E || !W || !E_out || !aligned16(E) || !aligned16(W) || !aligned16(E_out))
    return TINYKG_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace) || workspace_bytes < fwd_layout(g, d_in).total)
    return TINYKG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  switch (d_in) {
    case 32: return fwd_impl<32>(g, E, nullptr, nullptr, W, d_out, leaky_slope, bits, group, seed, E_out, saved, ws, st, true);
    case 64: return fwd_impl<64>(g, E, nullptr, nullptr, W, d_out, leaky_slope, bits, group, seed, E_out, saved, ws, st, true);
    case 128: return fwd_impl<128>(g, E, nullptr, nullptr, W, d_out, leaky_slope, bits, group, seed, E_out, saved, ws, st, true);
  }
  return TINYKG_ERR_UNSUPPORTED;
}

tinykg_status tinykg_kg_uniform_bwd(const tinykg_graph* g, const tinykg_saved* saved, const float* W,
                                    int d_in, int d_out, float leaky_slope, int bits, int group,
                                    const float* grad_E_out, float* grad_E, float* grad_W,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  using namespace tinykg;
  tinykg_status rc = check_common(g, d_in, d_in, d_out, bits, group);
  if (rc != TINYKG_OK) return rc;
  if ((rc = check_saved_uniform(saved, bits)) != TINYKG_OK) return rc;
  if (!W || !grad_W || !aligned16(W) || !aligned16(grad_W)) return TINYKG_ERR_INVALID_ARG;
  if (g->n_nodes > 0 && (!grad_E_out || !grad_E || !aligned16(grad_E_out) || !aligned16(grad_E)))
    return TINYKG_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace) || workspace_bytes < bwd_layout(g, d_in, d_out).total)
    return TINYKG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  switch (d_in) {
    case 32: return bwd_bits<32>(bits, g, saved, nullptr, nullptr, W, d_out, leaky_slope, group, grad_E_out, grad_E, nullptr, nullptr, grad_W, ws, st, true);
    case 64: return bwd_bits<64>(bits, g, saved, nullptr, nullptr, W, d_out, leaky_slope, group, grad_E_out, grad_E, nullptr, nullptr, grad_W, ws, st, true);
    case 128: return bwd_bits<128>(bits, g, saved, nullptr, nullptr, W, d_out, leaky_slope, group, grad_E_out, grad_E, nullptr, nullptr, grad_W, ws, st, true);
  }
  return TINYKG_ERR_UNSUPPORTED;
}

}  // extern "C"

// ------------------------------------------------ max-pooling aggregation (SPMM_MAX) ----
// M[h, c] = max over the out-edges (h, r, t) of E[t, c] (0 without out-edges).  What the
// backward pass needs is not an activation but, per output element, WHICH out-edge won: the
// context is that edge's number inside the head's neighbourhood (head order: relation, tail,
// input position; first one on ties), in the narrowest of 1 / 2 / 4 bytes that holds the
// graph's largest out-degree.  Backward: grad_E[t(arg), c] += grad_M[h, c].
namespace tinykg {

namespace {

template <typename ARG> struct ArgVec;
template <> struct ArgVec<uint8_t> { typedef uchar4 type; };
template <> struct ArgVec<uint16_t> { typedef ushort4 type; };
template <> struct ArgVec<uint32_t> { typedef uint4 type; };

// One LPR-lane slot per head for neighbourhoods of at most kSlotDegree edges (64 / LPR
// heads side by side), the whole wave for longer ones: its 64 / LPR lane groups take the
// edges j = sub, sub + ES, ... and their (value, number) pairs are merged at the end,
// larger value first, smaller number on equal values.
template <int D, typename ARG>
__global__ __launch_bounds__(kThreads) void max_fwd_kernel(const float* __restrict__ E,
                                                           const int32_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ h_tail, int64_t N,
                                                           float* __restrict__ M, ARG* __restrict__ arg) {
  constexpr int LPR = D / 4, ES = 64 / LPR;
  typedef typename ArgVec<ARG>::type AV;
  const int lane = threadIdx.x & 63;
  const int sub = lane / LPR, li = lane % LPR;
  const float4* rows = reinterpret_cast<const float4*>(E);
  const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
  auto take = [](float& best, uint32_t& at, float v, uint32_t j) {
    const bool win = v > best || (v == best && j < at);
    best = win ? v : best;
    at = win ? j : at;
  };
  auto store = [&](int64_t h, const float (&b)[4], const uint32_t (&a)[4]) {
    reinterpret_cast<float4*>(M)[h * LPR + li] = make_float4(b[0], b[1], b[2], b[3]);
    AV o;
    o.x = a[0]; o.y = a[1]; o.z = a[2]; o.w = a[3];
    reinterpret_cast<AV*>(arg)[h * LPR + li] = o;
  };
  for (int64_t h0 = ((int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)) * ES; h0 < N;
       h0 += n_waves * ES) {
    const int64_t h = h0 + sub;
    int e0 = 0, deg = 0;
    if (h < N) { e0 = rowptr[h]; deg = rowptr[h + 1] - e0; }
    const bool small = deg <= kSlotDegree;
    {
      const int ds = small ? deg : 0;
      float b[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      uint32_t a[4] = {0u, 0u, 0u, 0u};
      for (int j0 = 0; j0 < kSlotDegree; j0 += 4) {
        if (__builtin_amdgcn_ballot_w64(j0 < ds) == 0) break;
        float4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool on = j0 + u < ds;
          const int t = on ? h_tail[e0 + j0 + u] : 0;
          x[u] = rows[(int64_t)t * LPR + li];
          if (!on) x[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {       // in edge order with a strict comparison: the first maximum stays
          if (x[u].x > b[0]) { b[0] = x[u].x; a[0] = j0 + u; }
          if (x[u].y > b[1]) { b[1] = x[u].y; a[1] = j0 + u; }
          if (x[u].z > b[2]) { b[2] = x[u].z; a[2] = j0 + u; }
          if (x[u].w > b[3]) { b[3] = x[u].w; a[3] = j0 + u; }
        }
      }
      if (h < N && small) {
        if (deg == 0) { b[0] = b[1] = b[2] = b[3] = 0.f; }
        store(h, b, a);
      }
    }
    uint64_t pend = __builtin_amdgcn_ballot_w64(!small && li == 0);
    while (pend) {
      const int leader = __builtin_amdgcn_readfirstlane(__ffsll((long long)pend) - 1);
      pend &= pend - 1;
      const int64_t hw = h0 + leader / LPR;
      const int e0w = __builtin_amdgcn_readlane(e0, leader), degw = __builtin_amdgcn_readlane(deg, leader);
      float b[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      uint32_t a[4] = {0u, 0u, 0u, 0u};
      for (int base = 0; base < degw; base += 2 * ES) {
        const int j0 = base + sub, j1 = base + ES + sub;
        float4 x0 = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY), x1 = x0;
        if (j0 < degw) x0 = rows[(int64_t)h_tail[e0w + j0] * LPR + li];
        if (j1 < degw) x1 = rows[(int64_t)h_tail[e0w + j1] * LPR + li];
        if (x0.x > b[0]) { b[0] = x0.x; a[0] = j0; }
        if (x0.y > b[1]) { b[1] = x0.y; a[1] = j0; }
        if (x0.z > b[2]) { b[2] = x0.z; a[2] = j0; }
        if (x0.w > b[3]) { b[3] = x0.w; a[3] = j0; }
        if (x1.x > b[0]) { b[0] = x1.x; a[0] = j1; }
        if (x1.y > b[1]) { b[1] = x1.y; a[1] = j1; }
        if (x1.z > b[2]) { b[2] = x1.z; a[2] = j1; }
        if (x1.w > b[3]) { b[3] = x1.w; a[3] = j1; }
      }
      // merge the lane groups (lanes li, li + LPR, ...): xor steps LPR, 2 LPR, ..., 32
#pragma unroll
      for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float ov = __shfl_xor(b[c], o);
          const uint32_t oa = (uint32_t)__shfl_xor((int)a[c], o);
          take(b[c], a[c], ov, oa);
        }
      }
      if (sub == 0) store(hw, b, a);
    }
  }
}

__global__ __launch_bounds__(256) void max_bwd_zero_kernel(float* __restrict__ gE, int64_t n,
                                                           double* __restrict__ acc, int64_t m) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (int64_t i = i0; i < (n >> 2); i += stride) reinterpret_cast<float4*>(gE)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int64_t i = i0; i < m; i += stride) acc[i] = 0.0;
}

__global__ __launch_bounds__(256) void max_bwd_finish_kernel(HeavyFinish hf) {
  finish_heavy(hf, (int64_t)blockIdx.x * 256 + threadIdx.x, (int64_t)gridDim.x * 256);
}

int max_arg_bytes(const tinykg_graph* g) {
  return g->max_out_degree <= 256 ? 1 : g->max_out_degree <= 65536 ? 2 : 4;
}

template <int D, typename ARG>
tinykg_status max_fwd_impl(const tinykg_graph* g, const float* E, float* M, void* arg, hipStream_t st) {
  const int64_t N = g->n_nodes;
  const int wave_blocks = (int)std::max<int64_t>(1, std::min<int64_t>((N + 3) / 4, (int64_t)num_cus() * 16));
  ProfileScope prof("max_fwd_kernel", st);
  hipLaunchKernelGGL((max_fwd_kernel<D, ARG>), dim3(wave_blocks), dim3(kThreads), 0, st, E, g->rowptr, g->h_tail,
                     N, M, static_cast<ARG*>(arg));
  return launch_status();
}

template <int D, typename ARG>
tinykg_status max_bwd_impl(const tinykg_graph* g, const void* arg, const float* gM, float* gE, double* acc,
                           hipStream_t st) {
  const int64_t N = g->n_nodes;
  const int64_t n_heavy_elems = (int64_t)g->n_acc_heavy * D;
  const int zb = (int)std::min<int64_t>((N * D / 4 + 255) / 256, (int64_t)num_cus() * 8);
  ProfileScope prof("max_bwd_kernels", st);
  hipLaunchKernelGGL(max_bwd_zero_kernel, dim3(std::max(zb, 1)), dim3(256), 0, st, gE, N * D, acc,
                     n_heavy_elems * kHeavyReplicas);
  // the transposed walk of the uniform layer with another row: edges in (relation, tail)
  // order, 32 per wave, equal tails summed before one row of atomics per run
  if (g->n_edges > 0) {
    const GradSink sink{gE, acc, g->acc_slot};
    const int64_t waves = (g->n_edges + 31) / 32;
    const MaxRows<D, ARG> rows{g->rowptr, g->r_eid, gM, static_cast<const ARG*>(arg)};
    hipLaunchKernelGGL((uniform_bwd_kernel<D, MaxRows<D, ARG>>), dim3((unsigned)((waves + 3) / 4)), dim3(kThreads),
                       0, st, g->r_head, g->r_tail, g->r_hperm32, rows, g->n_edges, sink);
  }
  if (n_heavy_elems > 0) {
    const HeavyFinish hf{acc, g->acc_node, n_heavy_elems, D, gE};
    hipLaunchKernelGGL(max_bwd_finish_kernel, dim3(64), dim3(256), 0, st, hf);
  }
  return launch_status();
}

template <int D>
tinykg_status max_fwd_d(const tinykg_graph* g, const float* E, float* M, void* arg, hipStream_t st) {
  switch (max_arg_bytes(g)) {
    case 1: return max_fwd_impl<D, uint8_t>(g, E, M, arg, st);
    case 2: return max_fwd_impl<D, uint16_t>(g, E, M, arg, st);
  }
  return max_fwd_impl<D, uint32_t>(g, E, M, arg, st);
}
template <int D>
tinykg_status max_bwd_d(const tinykg_graph* g, const void* arg, const float* gM, float* gE, double* acc,
                        hipStream_t st) {
  switch (max_arg_bytes(g)) {
    case 1: return max_bwd_impl<D, uint8_t>(g, arg, gM, gE, acc, st);
    case 2: return max_bwd_impl<D, uint16_t>(g, arg, gM, gE, acc, st);
  }
  return max_bwd_impl<D, uint32_t>(g, arg, gM, gE, acc, st);
}

}  // namespace

}  // namespace tinykg

extern "C" {

int tinykg_kg_max_arg_bytes(const tinykg_graph* g) { return g ? tinykg::max_arg_bytes(g) : 0; }

size_t tinykg_kg_max_workspace_bytes(const tinykg_graph* g, int d) {
  using namespace tinykg;
  if (!g || !(d == 32 || d == 64 || d == 128)) return 0;
  return std::max<size_t>(256, (size_t)g->n_acc_heavy * kHeavyReplicas * d * sizeof(double));
}

tinykg_status tinykg_kg_max_fwd(const tinykg_graph* g, const float* E, int d, float* M, void* arg,
                                void* stream) {
  using namespace tinykg;
  if (!g) return TINYKG_ERR_INVALID_ARG;
  if (!(d == 32 || d == 64 || d == 128)) return TINYKG_ERR_UNSUPPORTED;
  if (g->n_nodes == 0) return TINYKG_OK;
  if (!E || !M || !arg || !aligned16(E) || !aligned16(M) || !aligned16(arg)) return TINYKG_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  switch (d) {
    case 32: return max_fwd_d<32>(g, E, M, arg, st);
    case 64: return max_fwd_d<64>(g, E, M, arg, st);
  }
  return max_fwd_d<128>(g, E, M, arg, st);
}

tinykg_status tinykg_kg_max_bwd(const tinykg_graph* g, const void* arg, int d, const float* grad_M,
                                float* grad_E, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace tinykg;
  if (!g) return TINYKG_ERR_INVALID_ARG;
  if (!(d == 32 || d == 64 || d == 128)) return TINYKG_ERR_UNSUPPORTED;
  if (g->n_nodes == 0) return TINYKG_OK;
  if (!arg || !grad_M || !grad_E || !aligned16(arg) || !aligned16(grad_M) || !aligned16(grad_E))
    return TINYKG_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace) || workspace_bytes < tinykg_kg_max_workspace_bytes(g, d))
    return TINYKG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  double* acc = static_cast<double*>(workspace);
  switch (d) {
    case 32: return max_bwd_d<32>(g, arg, grad_M, grad_E, acc, st);
    case 64: return max_bwd_d<64>(g, arg, grad_M, grad_E, acc, st);
  }
  return max_bwd_d<128>(g, arg, grad_M, grad_E, acc, st);
}

}  // extern "C"
