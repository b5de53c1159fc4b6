// Fused quantize + bit-pack and unpack + dequantize kernels for gfx950.
//
// Quant / Dequant are Eq. (3) / Eq. (4) of Sec. 3.3; the packed layout is the
// "bit-stream" of Sec. 4.1.4.  The exact arithmetic (operation order, rounding
// noise, packing order) is stated in include/tinykg.h.
//
// This file must be compiled with -ffp-contract=off: every float operation of
// the quantizer rounds once, in the order written.
//
// Kernel shape (quantize).  The path is bound by HBM reads (4 B/element in,
// bits/8 + 8/group out) only if the per-element VALU work stays small, so the
// layout is chosen to make each lane own 16 CONSECUTIVE elements:
//   * a wave streams tiles of 1024 elements; the four coalesced 128-bit loads
//     of a tile go through a wave-private 4 KiB LDS slab (XOR-swizzled so both
//     the row-wise write and the lane-contiguous read are bank-conflict free);
//   * 16 elements per lane means a group of G elements spans G/16 <= 16 lanes,
//     i.e. one DPP row: min/max finish with at most four DPP steps, and the two
//     IEEE divides (R/B, B/R) are paid once per 16 elements;
//   * one Philox4x32-10 block yields 8 x 16 random bits, so a lane needs exactly
//     two blocks, whose counters are (first_index + element)/8;
//   * the 16 codes of a lane are 16*bits contiguous bits of the stream: one
//     2/4/8/16-byte store per lane, contiguous across the wave.
// Every wave handles exactly one tile (grid = tiles / 4): blocks retire in address
// order, which keeps the DRAM access stream sequential.
#include "tinykg_common.h"

#include <float.h>

#include <type_traits>

namespace tinykg {

namespace {

// Streaming accesses: every input byte is read once and every output byte written once,
// so they are marked non-temporal (they should not displace anything from the caches).
typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4* p) {
  const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float4* p, const float4& v) {
  const floatx4 q = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(q, reinterpret_cast<floatx4*>(p));
}

constexpr int kWave = 64;
constexpr int kElemsPerLane = 16;
constexpr int kTileElems = kWave * kElemsPerLane;  // 1024 elements = 4 KiB of fp32
constexpr int kWavesPerBlock = 4;
constexpr int kTilesPerWave = 1;                   // consecutive tiles handled by one wave
constexpr int kBlock = kWave * kWavesPerBlock;

// ---- cross-lane exchange inside a DPP row (16 lanes) ------------------------
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kQuadSwap1 = 0xB1;   // quad_perm:[1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;   // quad_perm:[2,3,0,1]
constexpr int kHalfMirror = 0x141; // row_half_mirror
constexpr int kRowMirror = 0x140;  // row_mirror

// All-reduce over LPG (2,4,8,16) adjacent lanes: after each step the reduced
// sub-block is uniform, so mirroring pairs it with its neighbour sub-block.
template <int LPG>
__device__ __forceinline__ void group_minmax(float& mn, float& mx) {
  if (LPG >= 2) { mn = fminf(mn, dpp<kQuadSwap1>(mn)); mx = fmaxf(mx, dpp<kQuadSwap1>(mx)); }
  if (LPG >= 4) { mn = fminf(mn, dpp<kQuadSwap2>(mn)); mx = fmaxf(mx, dpp<kQuadSwap2>(mx)); }
  if (LPG >= 8) { mn = fminf(mn, dpp<kHalfMirror>(mn)); mx = fmaxf(mx, dpp<kHalfMirror>(mx)); }
  if (LPG >= 16) { mn = fminf(mn, dpp<kRowMirror>(mn)); mx = fmaxf(mx, dpp<kRowMirror>(mx)); }
}

__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c);
__device__ __forceinline__ uint32_t xnor3(uint32_t a, uint32_t b, uint32_t c);

// ---- Philox4x32-10 (Salmon et al., SC'11) -----------------------------------
// Counter (c0, c1, 0, 0), key (k0, k1).  The third and fourth counter words are
// zero by construction, which removes one multiply from the first round.
struct Philox4 { uint32_t w[4]; };

// COMPLEMENT: return the bitwise complement of the four output words (the two words
// that the last round produces by xor come out complemented at no cost).
template <bool COMPLEMENT>
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0,
                                                 uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)M0 * c0;
    const uint64_t p1 = (uint64_t)M1 * c2;
    const bool flip = COMPLEMENT && r == 9;
    const uint32_t n0 = flip ? xnor3((uint32_t)(p1 >> 32), c1, k0) : xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t n2 = flip ? xnor3((uint32_t)(p0 >> 32), c3, k1) : xor3((uint32_t)(p0 >> 32), c3, k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += W0;
    k1 += W1;
  }
  if (COMPLEMENT) { c1 = ~c1; c3 = ~c3; }
  return Philox4{{c0, c1, c2, c3}};
}

// Physical 16-byte slot of logical chunk `c` (0..255) of a wave's slab.  The
// owner lane of chunk c is i = c/4.  Only the low two bits are permuted, by
// s(i) = (bit2(i), bit1(i) ^ bit3(i)), so (a) consecutive chunks written by
// consecutive lanes still cover contiguous 64-byte runs, and (b) when every lane
// reads its j-th chunk, any 8 (or 16) neighbouring lanes touch 8 (or 16)
// different 16-byte bank groups.
__device__ __forceinline__ int slab_slot(int c) {
  const int s = ((c >> 3) & 2) | (((c >> 3) ^ (c >> 5)) & 1);
  return c ^ s;
}

// -ceil(X) as an integer in one instruction (floor of the negated operand).
__device__ __forceinline__ int neg_ceil_to_int(float X) {
  int r;
  asm("v_cvt_flr_i32_f32_e64 %0, -%1" : "=v"(r) : "v"(X));
  return r;
}

__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);   // a ^ b ^ c in one VALU op
}
__device__ __forceinline__ uint32_t xnor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x69);   // ~(a ^ b ^ c)
}

// (16-bit half HALF of w) - a, the half selected by the instruction's operand
// select (no separate mask / shift).
template <int HALF>
__device__ __forceinline__ uint32_t half_minus(uint32_t w, uint32_t a) {
  uint32_t r;
  if (HALF == 0)
    asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:DWORD"
        : "=v"(r) : "v"(w), "v"(a));
  else
    asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:DWORD"
        : "=v"(r) : "v"(w), "v"(a));
  return r;
}

// (S >> 16) << pos in one instruction (operand select picks the high half).
__device__ __forceinline__ uint32_t place_high_half(uint32_t S, uint32_t pos) {
  uint32_t r;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
      : "=v"(r) : "s"(pos), "v"(S));
  return r;
}

// Optional hook of the quantizer: it is shown every 128-bit chunk of an fp32 input as the
// kernel loaded it (index of the chunk in the flattened tensor, its column position, the four
// values), so that an operator which has to save Q(x) and also produce an elementwise
// function of x reads x once.  Chunk indices stay below 2^32 when a hook is active.
struct NoEpilogue {
  static constexpr bool kActive = false;
  uint32_t lpr = 1, step = 0;
  __device__ __forceinline__ void operator()(int64_t, uint32_t, const float4&) const {}
};

// y = (x - mu_c) a_c + beta_c per column c (the normalisation of a batch-norm layer whose
// input the same pass compresses).  lpr = chunks per row, step = 64 mod lpr.
struct AffineEpilogue {
  static constexpr bool kActive = true;
  uint32_t lpr, step;
  const float4* mu;
  const float4* a;
  const float4* beta;
  float4* y;
  __device__ __forceinline__ void operator()(int64_t c, uint32_t col, const float4& x) const {
    const float4 m = mu[col], s = a[col], b = beta[col];
    float4 o;
    o.x = fmaf(x.x - m.x, s.x, b.x); o.y = fmaf(x.y - m.y, s.y, b.y);
    o.z = fmaf(x.z - m.z, s.z, b.z); o.w = fmaf(x.w - m.w, s.w, b.w);
    store_stream(y + c, o);
  }
};

// IN = float: fp32 activations.  IN = uint16_t: bfloat16 activations (Sec. 4.1.4: half-precision
// inputs, for mixed-precision training); each value is widened to fp32 exactly and then takes
// the same path, so the output is that of the fp32 quantizer on the widened tensor.
template <typename IN, int BITS, int GROUP, int ROUNDING, typename EPI>
__global__ __launch_bounds__(kBlock) void quantize_kernel(
    const IN* __restrict__ act, int64_t n, uint32_t seed_lo, uint32_t seed_hi,
    uint64_t first_index, uint8_t* __restrict__ packed, float* __restrict__ gmin,
    float* __restrict__ gscale, EPI epi) {
  constexpr int LPG = GROUP / kElemsPerLane;       // lanes per group
  constexpr float Bf = (float)((1 << BITS) - 1);   // B = 2^b - 1
  constexpr float B16 = Bf * 65536.0f;
  constexpr int kWords = (kElemsPerLane * BITS + 31) / 32;

  __shared__ float4 slab[kWavesPerBlock][kTileElems / 4];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  float4* my = slab[wave];

  // kTilesPerWave consecutive tiles per wave; all their loads are issued up front
  constexpr bool kBf16 = std::is_same<IN, uint16_t>::value;
  const int64_t tile0 = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * kTilesPerWave;
  if (tile0 * kTileElems >= n) return;
  float4 v[kTilesPerWave][4];
  uint4 hv[kTilesPerWave][2];   // bf16: the lane's 16 elements are 32 contiguous bytes, loaded directly
#pragma unroll
  for (int tt = 0; tt < kTilesPerWave; ++tt) {
    if constexpr (kBf16) {
      const int64_t e = (tile0 + tt) * kTileElems + (int64_t)lane * kElemsPerLane;
      hv[tt][0] = make_uint4(0u, 0u, 0u, 0u); hv[tt][1] = hv[tt][0];
      if (e < n) {      // n and e are multiples of 16: the lane's 16 elements are all in range
        const floatx4* src = reinterpret_cast<const floatx4*>(act + e);
        const floatx4 q0 = __builtin_nontemporal_load(src), q1 = __builtin_nontemporal_load(src + 1);
        hv[tt][0] = make_uint4(__float_as_uint(q0.x), __float_as_uint(q0.y), __float_as_uint(q0.z), __float_as_uint(q0.w));
        hv[tt][1] = make_uint4(__float_as_uint(q1.x), __float_as_uint(q1.y), __float_as_uint(q1.z), __float_as_uint(q1.w));
      }
      continue;
    }
    const int64_t tile = tile0 + tt;
    const float4* src = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(act)) + tile * (kTileElems / 4) + lane;
    if ((tile + 1) * kTileElems <= n) {          // whole tile in range (wave-uniform)
#pragma unroll
      for (int u = 0; u < 4; ++u) v[tt][u] = load_stream(src + u * kWave);
    } else {
      const int64_t left = (n >> 2) - tile * (kTileElems / 4) - lane;   // chunks from `src` on
#pragma unroll
      for (int u = 0; u < 4; ++u)
        v[tt][u] = u * kWave < left ? load_stream(src + u * kWave) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }

#pragma unroll
  for (int tt = 0; tt < kTilesPerWave; ++tt) {
  const int64_t tile = tile0 + tt;
  if (tile * kTileElems >= n) break;
  const int64_t e0 = tile * kTileElems + (int64_t)lane * kElemsPerLane;  // lane's first element
  // stage the tile row-wise (coalesced order) into the swizzled slab
  float x[kElemsPerLane];
  if constexpr (kBf16) {
    const uint32_t w[8] = {hv[tt][0].x, hv[tt][0].y, hv[tt][0].z, hv[tt][0].w,
                           hv[tt][1].x, hv[tt][1].y, hv[tt][1].z, hv[tt][1].w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {       // bf16 -> fp32 is a 16-bit shift: exact
      x[2 * j + 0] = __uint_as_float(w[j] << 16);
      x[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
    }
  } else {
    // (slab_slot(u * 64 + lane) = u * 64 + slab_slot(lane): the swizzle only depends on
    // bits 3..5 of the chunk index and only changes bits 0..1)
    const int wslot = slab_slot(lane);
#pragma unroll
    for (int u = 0; u < 4; ++u) my[u * kWave + wslot] = v[tt][u];
    if constexpr (EPI::kActive) {
      const int64_t c0 = tile * (kTileElems / 4) + lane;
      uint32_t col = (uint32_t)c0 % epi.lpr;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (c0 + u * kWave < (n >> 2)) epi(c0 + u * kWave, col, v[tt][u]);
        col += epi.step;
        col = col >= epi.lpr ? col - epi.lpr : col;
      }
    }
    // lane-contiguous read-back: elements [16*lane, 16*lane+16) of the tile
    // (slab_slot(4 * lane + j) = slab_slot(4 * lane) ^ j for j < 4)
    const int rslot = slab_slot(4 * lane);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 r4 = my[rslot ^ j];
      x[4 * j + 0] = r4.x; x[4 * j + 1] = r4.y; x[4 * j + 2] = r4.z; x[4 * j + 3] = r4.w;
    }
  }
  const bool live = e0 < n;

  // Z = min, max of the group
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int j = 1; j < kElemsPerLane; ++j) { mn = fminf(mn, x[j]); mx = fmaxf(mx, x[j]); }
  group_minmax<LPG>(mn, mx);
  mn = mn + 0.0f;                       // -0 -> +0
  mx = mx + 0.0f;
  const float range = mx - mn;          // R
  // R / B and B / R (both correctly rounded) with ONE divide sequence: the even
  // lane of each pair computes R / B, the odd lane B / R, then they swap results
  // (a group always spans at least two lanes).
  const bool odd = lane & 1;
  const float q = (odd ? Bf : range) / (odd ? range : Bf);
  const float qs = dpp<kQuadSwap1>(q);
  const float scale = odd ? qs : q;     // R / B
  float inv = 0.0f;                     // B / R, kept finite; 0 for a constant group
  if (range > 0.0f) inv = fminf(odd ? q : qs, FLT_MAX);
  // (8-bit codes) an element equal to the group maximum gets code B by definition
  const float mxx = range > 0.0f ? mx : __builtin_nanf("");   // never matches if constant
  // rounding noise: two Philox blocks cover this lane's 16 elements.  What is
  // kept is 65535 - h (the complement of each 16-bit half).
  uint32_t nrnd[8];
  if (ROUNDING == TINYKG_ROUND_STOCHASTIC) {
    const uint64_t q = (first_index + (uint64_t)e0) >> 3;
    const Philox4 a = philox4x32_10<true>((uint32_t)q, (uint32_t)(q >> 32), seed_lo, seed_hi);
    const uint64_t q1 = q + 1;
    const Philox4 b = philox4x32_10<true>((uint32_t)q1, (uint32_t)(q1 >> 32), seed_lo, seed_hi);
#pragma unroll
    for (int i = 0; i < 4; ++i) { nrnd[i] = a.w[i]; nrnd[4 + i] = b.w[i]; }
  }

  // With X = xb * 2^16 (exact), floor(xb) + [h < frac(xb) * 2^16] equals
  // (ceil(X) + 65535 - h) >> 16, and nearest rounding is (floor(X) + 2^15) >> 16.
  uint32_t words[kWords];
  // SAFE: test every element against the maximum (needed for 8-bit codes, and for any
  // width when B/R overflowed and was clamped, which leaves R * inv far below B).
  auto encode = [&](auto safe_tag) {
    constexpr bool SAFE = decltype(safe_tag)::value;
#pragma unroll
    for (int w = 0; w < kWords; ++w) words[w] = 0u;
#pragma unroll
    for (int j = 0; j < kElemsPerLane; j += 2) {
      uint32_t placed[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float t = x[j + u] - mn;             // e - Z
        float X;
        if (!SAFE) {
          // The clamp alone implements both the clamp and the maximum rule when B <= 15 and
          // inv = fl(B/R): the maximum has t == R, and R * fl(B/R) is B or one of its two
          // neighbours.  One ulp above is clamped to B; one ulp below leaves a fractional
          // part of at least 1 - 2^-20, whose ceiling in 2^-16 units is a full step, so the
          // element rounds up to B for every noise value (and under nearest rounding).
          X = fminf((t * inv) * 65536.0f, B16);
        } else {
          const float xb = fminf(t * inv, Bf);     // (e - Z) / R * B, inside [0, B]
          X = xb * 65536.0f;
          X = (x[j + u] == mxx) ? B16 : X;
        }
        uint32_t S;                                // code in bits 16.., rubbish below
        if (ROUNDING == TINYKG_ROUND_STOCHASTIC) {
          const uint32_t a = (uint32_t)neg_ceil_to_int(X);
          S = u == 0 ? half_minus<0>(nrnd[j >> 1], a) : half_minus<1>(nrnd[j >> 1], a);
        } else {
          S = (uint32_t)X + 32768u;
        }
        placed[u] = place_high_half(S, ((j + u) * BITS) & 31);
      }
      words[(j * BITS) >> 5] |= placed[0] | placed[1];   // both land in the same word
    }
  };
  if (BITS <= 4 && __builtin_amdgcn_ballot_w64(inv == FLT_MAX) == 0) encode(std::false_type{});
  else encode(std::true_type{});

  if (live) {
    const int64_t bit0 = e0 * BITS;            // multiple of 16
    uint8_t* dst = packed + (bit0 >> 3);
    if (BITS == 1) {
      *reinterpret_cast<uint16_t*>(dst) = (uint16_t)words[0];
    } else if (BITS == 2) {
      *reinterpret_cast<uint32_t*>(dst) = words[0];
    } else if (BITS == 4) {
      *reinterpret_cast<uint2*>(dst) = make_uint2(words[0], words[kWords > 1 ? 1 : 0]);
    } else {
      *reinterpret_cast<uint4*>(dst) = make_uint4(words[0], words[kWords > 1 ? 1 : 0],
                                                  words[kWords > 2 ? 2 : 0],
                                                  words[kWords > 3 ? 3 : 0]);
    }
    if ((lane & (LPG - 1)) == 0) {
      const int64_t g = e0 / GROUP;
      gmin[g] = mn;
      gscale[g] = scale;
    }
  }
  }  // tiles of this wave
}

// ---- unpack + dequantize ------------------------------------------------------
// A block owns kDqU * 256 consecutive 128-bit output chunks; thread t handles
// chunks t, t+256, ... of it, so every load and store instruction of a wave is
// contiguous.  All loads of a thread are issued before its first store, and each
// thread reads only the 4*bits bits a chunk needs.
constexpr int kDqU = 4;

template <int BITS>
__device__ __forceinline__ uint32_t load_codes4(const uint8_t* __restrict__ packed, int64_t c) {
  if (BITS == 8) return reinterpret_cast<const uint32_t*>(packed)[c];
  if (BITS == 4) return reinterpret_cast<const uint16_t*>(packed)[c];
  if (BITS == 2) return packed[c];
  return (packed[c >> 1] >> ((c & 1) * 4)) & 0xFu;
}

template <int BITS>
__global__ __launch_bounds__(256) void dequantize_kernel(
    const uint8_t* __restrict__ packed, const float* __restrict__ gmin,
    const float* __restrict__ gscale, int64_t n_chunks, int group_chunks_log2,
    float* __restrict__ out) {
  constexpr uint32_t B = (1u << BITS) - 1u;
  const int64_t c0 = (int64_t)blockIdx.x * (256 * kDqU) + threadIdx.x;
  uint32_t w[kDqU];
  float z[kDqU], s[kDqU];
#pragma unroll
  for (int u = 0; u < kDqU; ++u) {
    const int64_t c = c0 + u * 256;
    w[u] = 0; z[u] = 0.f; s[u] = 0.f;
    if (c < n_chunks) {
      w[u] = load_codes4<BITS>(packed, c);
      const int64_t g = c >> group_chunks_log2;
      z[u] = gmin[g];
      s[u] = gscale[g];
    }
  }
#pragma unroll
  for (int u = 0; u < kDqU; ++u) {
    const int64_t c = c0 + u * 256;
    if (c < n_chunks) {
      float4 v;
      v.x = fmaf((float)(w[u] & B), s[u], z[u]);
      v.y = fmaf((float)((w[u] >> BITS) & B), s[u], z[u]);
      v.z = fmaf((float)((w[u] >> (2 * BITS)) & B), s[u], z[u]);
      v.w = fmaf((float)((w[u] >> (3 * BITS)) & B), s[u], z[u]);
      store_stream(reinterpret_cast<float4*>(out) + c, v);
    }
  }
}

int ilog2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

template <typename IN, int BITS, int ROUNDING, typename EPI = NoEpilogue>
tinykg_status launch_quantize_g(const IN* act, int64_t n, int group, uint64_t seed,
                                uint64_t first_index, uint8_t* packed, float* gmin, float* gscale,
                                hipStream_t stream, EPI epi = EPI{}) {
  const int64_t n_tiles = (n + kTileElems - 1) / kTileElems;
  const int64_t per_block = kWavesPerBlock * kTilesPerWave;
  const int64_t want = (n_tiles + per_block - 1) / per_block;
  if (want >= ((int64_t)1 << 31)) return TINYKG_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)want);
  const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
  ProfileScope prof("quantize_kernel", stream);
#define TINYKG_Q_LAUNCH(G)                                                                   \
  hipLaunchKernelGGL((quantize_kernel<IN, BITS, G, ROUNDING, EPI>), grid, dim3(kBlock), 0, stream, act, n, \
                     lo, hi, first_index, packed, gmin, gscale, epi)
  switch (group) {
    case 32: TINYKG_Q_LAUNCH(32); break;
    case 64: TINYKG_Q_LAUNCH(64); break;
    case 128: TINYKG_Q_LAUNCH(128); break;
    case 256: TINYKG_Q_LAUNCH(256); break;
    default: return TINYKG_ERR_INVALID_ARG;
  }
#undef TINYKG_Q_LAUNCH
  return launch_status();
}

template <typename IN, int ROUNDING>
tinykg_status launch_quantize_b(const IN* act, int64_t n, int bits, int group, uint64_t seed,
                                uint64_t first_index, uint8_t* packed, float* gmin, float* gscale,
                                hipStream_t stream) {
  switch (bits) {
    case 1: return launch_quantize_g<IN, 1, ROUNDING>(act, n, group, seed, first_index, packed, gmin, gscale, stream);
    case 2: return launch_quantize_g<IN, 2, ROUNDING>(act, n, group, seed, first_index, packed, gmin, gscale, stream);
    case 4: return launch_quantize_g<IN, 4, ROUNDING>(act, n, group, seed, first_index, packed, gmin, gscale, stream);
    case 8: return launch_quantize_g<IN, 8, ROUNDING>(act, n, group, seed, first_index, packed, gmin, gscale, stream);
    default: return TINYKG_ERR_INVALID_ARG;
  }
}

}  // namespace

int num_cus() {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0)
      cus = 256;
    cached = cus;
  }
  return cached;
}

template <typename IN>
tinykg_status launch_quantize_any(const IN* act, int64_t n, int bits, int group, uint64_t seed,
                                  uint64_t first_index, int rounding, uint8_t* packed, float* gmin,
                                  float* gscale, hipStream_t stream) {
  if (!bits_ok(bits) || !group_ok(group)) return TINYKG_ERR_INVALID_ARG;
  if (rounding != TINYKG_ROUND_STOCHASTIC && rounding != TINYKG_ROUND_NEAREST)
    return TINYKG_ERR_INVALID_ARG;
  if (n < 0 || n % group != 0 || first_index % (uint64_t)group != 0) return TINYKG_ERR_SHAPE;
  if (n == 0) return TINYKG_OK;
  if (!act || !packed || !gmin || !gscale) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(act) || !aligned16(packed) || !aligned16(gmin) || !aligned16(gscale))
    return TINYKG_ERR_INVALID_ARG;
  if (rounding == TINYKG_ROUND_STOCHASTIC)
    return launch_quantize_b<IN, TINYKG_ROUND_STOCHASTIC>(act, n, bits, group, seed, first_index,
                                                          packed, gmin, gscale, stream);
  return launch_quantize_b<IN, TINYKG_ROUND_NEAREST>(act, n, bits, group, seed, first_index, packed,
                                                     gmin, gscale, stream);
}

tinykg_status launch_quantize(const float* act, int64_t n, int bits, int group, uint64_t seed,
                              uint64_t first_index, int rounding, uint8_t* packed, float* gmin,
                              float* gscale, hipStream_t stream) {
  return launch_quantize_any<float>(act, n, bits, group, seed, first_index, rounding, packed, gmin,
                                    gscale, stream);
}

tinykg_status launch_quantize_affine(const float* act, int64_t n, int bits, int group, uint64_t seed,
                                     uint8_t* packed, float* gmin, float* gscale, int dim,
                                     const float* mu, const float* a, const float* beta, float* y,
                                     hipStream_t stream) {
  if (!bits_ok(bits) || !group_ok(group)) return TINYKG_ERR_INVALID_ARG;
  if (n <= 0 || n % group != 0 || dim < 4 || dim % 4 != 0 || (n >> 2) >= ((int64_t)1 << 32))
    return TINYKG_ERR_SHAPE;
  AffineEpilogue epi;
  epi.lpr = (uint32_t)(dim / 4);
  epi.step = 64u % epi.lpr;
  epi.mu = reinterpret_cast<const float4*>(mu);
  epi.a = reinterpret_cast<const float4*>(a);
  epi.beta = reinterpret_cast<const float4*>(beta);
  epi.y = reinterpret_cast<float4*>(y);
  constexpr int RS = TINYKG_ROUND_STOCHASTIC;
  switch (bits) {
    case 1: return launch_quantize_g<float, 1, RS, AffineEpilogue>(act, n, group, seed, 0, packed, gmin, gscale, stream, epi);
    case 2: return launch_quantize_g<float, 2, RS, AffineEpilogue>(act, n, group, seed, 0, packed, gmin, gscale, stream, epi);
    case 4: return launch_quantize_g<float, 4, RS, AffineEpilogue>(act, n, group, seed, 0, packed, gmin, gscale, stream, epi);
    case 8: return launch_quantize_g<float, 8, RS, AffineEpilogue>(act, n, group, seed, 0, packed, gmin, gscale, stream, epi);
  }
  return TINYKG_ERR_INVALID_ARG;
}

tinykg_status launch_dequantize(const uint8_t* packed, const float* gmin, const float* gscale,
                                int64_t n, int bits, int group, float* out, hipStream_t stream) {
  if (!bits_ok(bits) || !group_ok(group)) return TINYKG_ERR_INVALID_ARG;
  if (n < 0 || n % group != 0) return TINYKG_ERR_SHAPE;
  if (n == 0) return TINYKG_OK;
  if (!packed || !gmin || !gscale || !out) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(packed) || !aligned16(gmin) || !aligned16(gscale) || !aligned16(out))
    return TINYKG_ERR_INVALID_ARG;
  const int64_t n_chunks = n >> 2;
  const int64_t want = (n_chunks + 256 * kDqU - 1) / (256 * kDqU);
  if (want >= ((int64_t)1 << 31)) return TINYKG_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)want);
  const int gl2 = ilog2(group / 4);
  ProfileScope prof("dequantize_kernel", stream);
#define TINYKG_DQ_LAUNCH(BITS)                                                              \
  hipLaunchKernelGGL((dequantize_kernel<BITS>), grid, dim3(256), 0, stream, packed, gmin, gscale, \
                     n_chunks, gl2, out)
  switch (bits) {
    case 1: TINYKG_DQ_LAUNCH(1); break;
    case 2: TINYKG_DQ_LAUNCH(2); break;
    case 4: TINYKG_DQ_LAUNCH(4); break;
    default: TINYKG_DQ_LAUNCH(8); break;
  }
#undef TINYKG_DQ_LAUNCH
  return launch_status();
}

}  // namespace tinykg

extern "C" {

const char* tinykg_status_string(tinykg_status s) {
  switch (s) {
    case TINYKG_OK: return "ok";
    case TINYKG_ERR_INVALID_ARG: return "invalid argument";
    case TINYKG_ERR_SHAPE: return "shape mismatch";
    case TINYKG_ERR_UNSUPPORTED: return "unsupported size";
    case TINYKG_ERR_WORKSPACE: return "workspace too small";
    case TINYKG_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

size_t tinykg_packed_bytes(int64_t rows, int64_t dim, int bits) {
  if (rows < 0 || dim < 0 || bits <= 0) return 0;
  return (size_t)(((unsigned __int128)rows * (unsigned __int128)dim * (unsigned)bits + 7) / 8);
}

int64_t tinykg_num_groups(int64_t rows, int64_t dim, int group) {
  if (rows < 0 || dim < 0 || group <= 0) return 0;
  return rows * dim / group;
}

tinykg_status tinykg_quantize_ex(const float* act, int64_t rows, int64_t dim, int bits, int group,
                                 uint64_t seed, uint64_t first_index, int rounding,
                                 uint8_t* packed, float* gmin, float* gscale, void* stream) {
  if (rows < 0 || dim < 0) return TINYKG_ERR_SHAPE;
  if (rows != 0 && dim > INT64_MAX / rows) return TINYKG_ERR_SHAPE;
  return tinykg::launch_quantize(act, rows * dim, bits, group, seed, first_index, rounding, packed,
                                 gmin, gscale, (hipStream_t)stream);
}

tinykg_status tinykg_quantize(const float* act, int64_t rows, int64_t dim, int bits, int group,
                              uint64_t seed, uint8_t* packed, float* gmin, float* gscale,
                              void* stream) {
  return tinykg_quantize_ex(act, rows, dim, bits, group, seed, 0, TINYKG_ROUND_STOCHASTIC, packed,
                            gmin, gscale, stream);
}

tinykg_status tinykg_quantize_bf16(const uint16_t* act, int64_t rows, int64_t dim, int bits,
                                   int group, uint64_t seed, uint64_t first_index, int rounding,
                                   uint8_t* packed, float* gmin, float* gscale, void* stream) {
  if (rows < 0 || dim < 0) return TINYKG_ERR_SHAPE;
  if (rows != 0 && dim > INT64_MAX / rows) return TINYKG_ERR_SHAPE;
  return tinykg::launch_quantize_any<uint16_t>(act, rows * dim, bits, group, seed, first_index,
                                               rounding, packed, gmin, gscale, (hipStream_t)stream);
}

tinykg_status tinykg_dequantize(const uint8_t* packed, const float* gmin, const float* gscale,
                                int64_t rows, int64_t dim, int bits, int group, float* out,
                                void* stream) {
  if (rows < 0 || dim < 0) return TINYKG_ERR_SHAPE;
  if (rows != 0 && dim > INT64_MAX / rows) return TINYKG_ERR_SHAPE;
  return tinykg::launch_dequantize(packed, gmin, gscale, rows * dim, bits, group, out,
                                   (hipStream_t)stream);
}

}  // extern "C"
