// CPU oracle for the TinyKG activation compressor.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain, obviously-correct statement of what the
// compressor computes.  It exists so that the GPU library can be checked
// against it; nothing in the product path may include, link or call it, and it
// shares no code, header, table or helper with the GPU sources.
//
// What it follows (TinyKG, RecSys'22):
//   * Quant    -- Sec. 3.3 "Quantization (Float -> Integer)", Eq. (3):
//                 code = SR( (e - Z) / R * B ),  B = 2^b - 1,
//                 Z = min, R = max - min of the group, SR = stochastic rounding
//                 (up with probability equal to the fractional part).
//   * Dequant  -- Sec. 3.3 "Dequantization (Integer -> Float)", Eq. (4):
//                 e_hat = R * code / B + Z.
//   * Bit-streams -- Sec. 4.1.4: codes narrower than a byte are stored as a
//                 packed bit-stream.
// Readings where the paper is silent (all stated again where they are used):
//   groups are runs of G consecutive elements of the row-major flattened
//   tensor; the stored pair is (min, scale = R/B); the random numbers come from
//   Philox4x32-10 (Salmon et al., SC'11) keyed by the seed with the element
//   index as counter, 16 bits per element; codes are packed LSB-first.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -shared -fPIC (no fast-math; every
// float operation below rounds exactly once, in the order written).
//
// Parity pins for this file live in tests/test_oracle_quant.py.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

namespace {

// ---- Philox4x32-10, written from the round definition in Salmon et al. -----
// One round maps (c0,c1,c2,c3) under round key (k0,k1) to
//   (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0)),
// with M0 = 0xD2511F53, M1 = 0xCD9E8D57; between rounds the key is advanced by
// the Weyl constants (0x9E3779B9, 0xBB67AE85).
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint64_t p0 = M0 * (uint64_t)c0;
    const uint64_t p1 = M1 * (uint64_t)c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 16 random bits for flat element index i under `seed`.
// Reading: one Philox block serves 8 consecutive elements; block number i/8 is
// the (64-bit) counter, the seed is the (64-bit) key; element i takes the low
// half (i even) or the high half (i odd) of output word (i/2) mod 4.
uint32_t noise16(uint64_t seed, uint64_t i) {
  const uint64_t q = i >> 3;
  const uint32_t ctr[4] = {(uint32_t)q, (uint32_t)(q >> 32), 0u, 0u};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t o[4];
  philox4x32_10(ctr, key, o);
  const uint32_t w = o[(i >> 1) & 3];
  return (i & 1) ? (w >> 16) : (w & 0xFFFFu);
}

bool bits_ok(int bits) { return bits == 1 || bits == 2 || bits == 4 || bits == 8; }

}  // namespace

extern "C" {

// Raw generator, exposed so tests can check it against published known answers.
void tinykg_ref_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

uint32_t tinykg_ref_noise16(uint64_t seed, uint64_t index) { return noise16(seed, index); }

// Bit-stream packing (Sec. 4.1.4).  Reading: element i occupies bits
// [(i*b) mod 8, (i*b) mod 8 + b) of byte (i*b)/8, least-significant first, no
// padding.  `packed` must hold n*bits/8 bytes (n*bits divisible by 8).
int tinykg_ref_pack(const uint8_t* codes, int64_t n, int bits, uint8_t* packed) {
  if (!bits_ok(bits) || n < 0 || (n * bits) % 8 != 0) return 1;
  std::memset(packed, 0, (size_t)(n * bits / 8));
  for (int64_t i = 0; i < n; ++i) {
    if (codes[i] >> bits) return 1;  // code does not fit
    const int64_t bitpos = i * bits;
    packed[bitpos >> 3] |= (uint8_t)(codes[i] << (bitpos & 7));
  }
  return 0;
}

int tinykg_ref_unpack(const uint8_t* packed, int64_t n, int bits, uint8_t* codes) {
  if (!bits_ok(bits) || n < 0) return 1;
  const uint32_t B = (1u << bits) - 1u;
  for (int64_t i = 0; i < n; ++i) {
    const int64_t bitpos = i * bits;
    codes[i] = (uint8_t)((packed[bitpos >> 3] >> (bitpos & 7)) & B);
  }
  return 0;
}

// Quant of Eq. (3) on n = rows*dim elements whose flat indices in the full
// tensor are first_index .. first_index+n-1 (first_index lets a test quantize a
// slice of a large tensor and get the bytes the full run would produce; it must
// be a multiple of the group size).  rounding: 0 = stochastic, 1 = nearest.
// Writes the unpacked codes (one per byte), the per-group minimum and scale.
int tinykg_ref_quantize_codes(const float* act, int64_t n, int bits, int group, uint64_t seed,
                              uint64_t first_index, int rounding, uint8_t* codes, float* gmin,
                              float* gscale) {
  if (!bits_ok(bits) || group <= 0 || n < 0 || n % group != 0) return 1;
  if (first_index % (uint64_t)group != 0) return 1;
  const float Bf = (float)((1 << bits) - 1);  // number of bins B = 2^b - 1
  for (int64_t g = 0; g < n / group; ++g) {
    const float* x = act + g * group;
    // Z = min, max over the group (exact, order-free).
    float mn = x[0], mx = x[0];
    for (int j = 1; j < group; ++j) {
      if (x[j] < mn) mn = x[j];
      if (x[j] > mx) mx = x[j];
    }
    mn = mn + 0.0f;  // reading: a minimum of -0 is stored as +0 ...
    mx = mx + 0.0f;  // ... and likewise the maximum, so R and R/B of an all-zero
                     // group are +0 whatever the order of its +0 / -0 elements
    const float range = mx - mn;       // R, rounded once
    const float scale = range / Bf;    // R / B, correctly rounded
    // B / R, correctly rounded.  Reading: when R is so small that B/R is not
    // finite the factor is the largest finite float, so that 0 * factor stays 0.
    float inv = 0.0f;
    if (range > 0.0f) {
      inv = Bf / range;
      if (inv > std::numeric_limits<float>::max()) inv = std::numeric_limits<float>::max();
    }
    gmin[g] = mn;
    gscale[g] = scale;
    for (int j = 0; j < group; ++j) {
      const float t = x[j] - mn;           // e - Z
      float xb = t * inv;                  // (e - Z) / R * B
      if (!(xb < Bf)) xb = Bf;             // stays inside [0, B]
      const float f = std::floor(xb);
      const float p = xb - f;              // fractional part, exact
      int code;
      if (rounding == 0) {
        // up with probability p: compare p with a 16-bit uniform h / 2^16
        const uint32_t h = noise16(seed, first_index + (uint64_t)(g * group + j));
        code = (int)f + (((float)h < p * 65536.0f) ? 1 : 0);
      } else {
        code = (int)f + ((p >= 0.5f) ? 1 : 0);
      }
      // Reading: the group maximum is code B by definition (in real arithmetic
      // (max - Z)/R*B = B; in float the product can fall one ulp short).
      if (x[j] == mx && range > 0.0f) code = (int)Bf;
      codes[g * group + j] = (uint8_t)code;
    }
  }
  return 0;
}

// Quant + bit-stream: the compressor's forward half.
int tinykg_ref_quantize(const float* act, int64_t rows, int64_t dim, int bits, int group,
                        uint64_t seed, uint64_t first_index, int rounding, uint8_t* packed,
                        float* gmin, float* gscale) {
  if (rows < 0 || dim < 0) return 1;
  const int64_t n = rows * dim;
  if (n == 0) return bits_ok(bits) && group > 0 ? 0 : 1;
  uint8_t* codes = new uint8_t[(size_t)n];
  int rc = tinykg_ref_quantize_codes(act, n, bits, group, seed, first_index, rounding, codes, gmin,
                                     gscale);
  if (rc == 0) rc = tinykg_ref_pack(codes, n, bits, packed);
  delete[] codes;
  return rc;
}

// Dequant of Eq. (4): e_hat = code * (R/B) + Z.  Reading: evaluated as one
// fused multiply-add (a single rounding).
int tinykg_ref_dequantize(const uint8_t* packed, const float* gmin, const float* gscale,
                          int64_t rows, int64_t dim, int bits, int group, float* out) {
  if (!bits_ok(bits) || group <= 0 || rows < 0 || dim < 0) return 1;
  const int64_t n = rows * dim;
  if (n % group != 0) return 1;
  const uint32_t B = (1u << bits) - 1u;
  for (int64_t i = 0; i < n; ++i) {
    const int64_t bitpos = i * bits;
    const uint32_t code = (packed[bitpos >> 3] >> (bitpos & 7)) & B;
    out[i] = std::fmaf((float)code, gscale[i / group], gmin[i / group]);
  }
  return 0;
}

}  // extern "C"
