// Driver for the sanitizer build of the CPU oracle (test infrastructure): calls every entry
// point of oracle/tinykg_ref_quant.cpp and oracle/tinykg_ref_agg.cpp once on small seeded
// inputs -- all bit widths, a ragged unpack, a slice with first_index, a graph with a
// head without edges, repeated triplets and a self-loop -- so that AddressSanitizer and
// UndefinedBehaviorSanitizer see each loop's first and last iteration.  Prints "ok".
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
void tinykg_ref_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out);
int tinykg_ref_pack(const uint8_t* codes, int64_t n, int bits, uint8_t* packed);
int tinykg_ref_unpack(const uint8_t* packed, int64_t n, int bits, uint8_t* codes);
int tinykg_ref_quantize(const float* act, int64_t rows, int64_t dim, int bits, int group,
                        uint64_t seed, uint64_t first_index, int rounding, uint8_t* packed,
                        float* gmin, float* gscale);
int tinykg_ref_dequantize(const uint8_t* packed, const float* gmin, const float* gscale,
                          int64_t rows, int64_t dim, int bits, int group, float* out);
int tinykg_ref_kg_aggregate_fwd(int64_t N, int R, int64_t T, const int32_t* head,
                                const int32_t* rel, const int32_t* tail, const float* E,
                                const float* Wr, const float* er, const float* W, int d, int k,
                                int dout, float slope, int threads, float* Eout, float* H,
                                uint8_t* mask_out);
int tinykg_ref_kg_aggregate_bwd(int64_t N, int R, int64_t T, const int32_t* head,
                                const int32_t* rel, const int32_t* tail, const float* Ehat,
                                const float* Hhat, const uint8_t* mask, const float* Wr,
                                const float* er, const float* W, int d, int k, int dout,
                                float slope, const float* gEout, int threads, float* gE,
                                float* gWr, float* ger, float* gW);
}

namespace {
uint64_t state = 0x9E3779B97F4A7C15ull;
float next_unit() {   // xorshift64*, mapped to [-1, 1)
  state ^= state >> 12; state ^= state << 25; state ^= state >> 27;
  const uint64_t r = state * 0x2545F4914F6CDD1Dull;
  return (float)((double)(r >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
std::vector<float> draw(size_t n, float scale) {
  std::vector<float> v(n);
  for (auto& x : v) x = scale * next_unit();
  return v;
}
#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "failed: %s (line %d)\n", #cond, __LINE__); return 1; } } while (0)
}  // namespace

int main() {
  uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
  tinykg_ref_philox4x32_10(ctr, key, out);

  const int64_t rows = 24, dim = 32;
  const auto x = draw((size_t)(rows * dim), 3.0f);
  for (int bits : {1, 2, 4, 8}) {
    for (int group : {32, 64, 128, 256}) {
      const int64_t n = rows * dim;
      std::vector<uint8_t> packed((size_t)(n * bits / 8));
      std::vector<float> mn((size_t)(n / group)), sc((size_t)(n / group)), back((size_t)n);
      for (int rounding : {0, 1}) {
        CHECK(tinykg_ref_quantize(x.data(), rows, dim, bits, group, 7, 0, rounding, packed.data(), mn.data(), sc.data()) == 0);
        CHECK(tinykg_ref_dequantize(packed.data(), mn.data(), sc.data(), rows, dim, bits, group, back.data()) == 0);
      }
      // a slice of a larger tensor: the counter starts at first_index (also beyond 2^35)
      CHECK(tinykg_ref_quantize(x.data() + 256, (n - 256) / dim, dim, bits, group, 7, ((uint64_t)1 << 35) + 256, 0,
                                packed.data(), mn.data(), sc.data()) == 0);
    }
    // pack 16 codes (whole bytes at every width), unpack a ragged prefix of 13
    std::vector<uint8_t> codes(16), pk((size_t)(16 * bits / 8)), un(13);
    for (size_t i = 0; i < codes.size(); ++i) codes[i] = (uint8_t)(i & ((1u << bits) - 1u));
    CHECK(tinykg_ref_pack(codes.data(), 16, bits, pk.data()) == 0);
    CHECK(tinykg_ref_unpack(pk.data(), 13, bits, un.data()) == 0);
    for (size_t i = 0; i < un.size(); ++i) CHECK(codes[i] == un[i]);
  }
  CHECK(tinykg_ref_quantize(x.data(), 0, dim, 2, 64, 1, 0, 0, nullptr, nullptr, nullptr) == 0);

  // aggregation: 9 nodes (node 8 has no out-edge), 3 relations, repeated triplets, a self-loop
  const int64_t N = 9, T = 14;
  const int R = 3, d = 8, dout = 16;
  const int32_t head[T] = {0, 0, 0, 1, 1, 2, 3, 3, 4, 5, 6, 7, 7, 0};
  const int32_t rel[T]  = {0, 1, 2, 0, 0, 1, 2, 2, 0, 1, 2, 0, 1, 0};
  const int32_t tail[T] = {1, 2, 3, 1, 1, 0, 8, 8, 8, 4, 5, 6, 7, 1};
  const auto E = draw((size_t)(N * d), 0.5f), Wr = draw((size_t)(R * d * d), 0.4f), er = draw((size_t)(R * d), 0.2f),
             W = draw((size_t)(dout * d), 0.4f), G = draw((size_t)(N * dout), 1.0f);
  for (int threads : {1, 3}) {
    std::vector<float> Eo((size_t)(N * dout)), H((size_t)(N * d)), gE((size_t)(N * d)), gWr((size_t)(R * d * d)),
        ger((size_t)(R * d)), gW((size_t)(dout * d));
    std::vector<uint8_t> mask((size_t)(N * dout));
    CHECK(tinykg_ref_kg_aggregate_fwd(N, R, T, head, rel, tail, E.data(), Wr.data(), er.data(), W.data(), d, d, dout,
                                      0.2f, threads, Eo.data(), H.data(), mask.data()) == 0);
    CHECK(tinykg_ref_kg_aggregate_bwd(N, R, T, head, rel, tail, E.data(), H.data(), mask.data(), Wr.data(), er.data(),
                                      W.data(), d, d, dout, 0.2f, G.data(), threads, gE.data(), gWr.data(), ger.data(),
                                      gW.data()) == 0);
  }
  // no edges at all
  {
    std::vector<float> Eo((size_t)(N * dout)), H((size_t)(N * d));
    std::vector<uint8_t> mask((size_t)(N * dout));
    CHECK(tinykg_ref_kg_aggregate_fwd(N, R, 0, head, rel, tail, E.data(), Wr.data(), er.data(), W.data(), d, d, dout,
                                      0.2f, 2, Eo.data(), H.data(), mask.data()) == 0);
  }
  std::puts("ok");
  return 0;
}
