// Driver for the sanitizer run of the CPU oracle (tests/test_oracle_sanitizers.py builds it together
// with oracle/hago_ref.cpp under -fsanitize=address,undefined and expects a clean exit).  It calls
// every oracle entry point on inputs chosen to reach the arithmetic's edges: INT32 extremes through
// every shift, wrapping sums, padded taps, NaN / infinite / huge reals, empty tensors.  Tensors are
// heap arrays of exactly the stated size, so any out-of-bounds access is reported.
#include "../oracle/hago_ref.h"

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <vector>

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "driver: %s failed at line %d\n", #c, __LINE__); std::exit(2); } } while (0)

static uint64_t rng_state = 0x4841474full;
static uint32_t rnd() {  // SplitMix64
  uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return (uint32_t)((z ^ (z >> 31)) >> 16);
}

int main() {
  const int32_t i32min = std::numeric_limits<int32_t>::min(), i32max = std::numeric_limits<int32_t>::max();
  // requantize: extremes through every shift and both tie rules, multiplier at both ends of its range
  const int32_t accs[] = {i32min, i32min + 1, -1, 0, 1, i32max - 1, i32max, 1 << 30, -(1 << 30)};
  const int32_t mults[] = {1 << 30, (1 << 30) + 1, i32max};
  for (int32_t a : accs)
    for (int sh = 0; sh <= 31; ++sh)
      for (int rd = 0; rd <= 1; ++rd) {
        for (int32_t m : mults) {
          const int64_t v = hago_ref_requantize_one_mode(a, m, sh, 255, i32min, i32max, rd);
          REQUIRE(v >= (int64_t)i32min && v <= (int64_t)i32max);
        }
        const int64_t s = hago_ref_requantize_shift_one(a, sh, -256, i32min, i32max, rd);
        REQUIRE(s >= (int64_t)i32min && s <= (int64_t)i32max);
      }
  int32_t m = 0, sh = 0;
  REQUIRE(hago_ref_encode_multiplier(0.1, &m, &sh) == REF_OK && m == 1717986918 && sh == 3);
  REQUIRE(hago_ref_encode_multiplier(1.0 - 1e-12, &m, &sh) != REF_OK);
  REQUIRE(hago_ref_encode_multiplier(std::ldexp(1.0, -33), &m, &sh) != REF_OK);
  REQUIRE(hago_ref_encode_multiplier(std::nan(""), &m, &sh) != REF_OK);
  REQUIRE(hago_ref_scale(4.0, 8, 1) == 4.0 / 128.0);
  int32_t lo = 0, hi = 0;
  REQUIRE(hago_ref_bit_range(31, 1, &lo, &hi) == REF_OK && lo == -(1 << 30) && hi == (1 << 30) - 1);
  REQUIRE(hago_ref_bit_range(31, 0, &lo, &hi) == REF_OK && hi == i32max);
  REQUIRE(hago_ref_acc16_safe(312, 15, 7) == 1 && hago_ref_acc_safe(521, 127, 127, 24) == 0);
  REQUIRE(hago_ref_acc_safe(i32max, i32max, i32max, 32) == 0);

  // elementwise operators on the awkward reals
  const int64_t O = 2, C = 3, I = 7, n = O * C * I;
  std::vector<float> x(n), y(n), thr(C);
  const float specials[] = {0.0f, -0.0f, 0.5f, -0.5f, 1e30f, -1e30f, INFINITY, -INFINITY, NAN, 1e-42f, 3.4e38f, -2.5f};
  for (int64_t i = 0; i < n; ++i) x[i] = specials[i % 12] + (float)(i / 12);
  std::vector<float> scale = {0.25f, 1e-30f, 3.0e38f};
  std::vector<int32_t> zp = {0, 128, -7}, q(n);
  REQUIRE(hago_ref_simquant(x.data(), y.data(), O, C, I, scale.data(), zp.data(), 1, -128, 127) == REF_OK);
  REQUIRE(hago_ref_simquant(x.data(), y.data(), O, C, I, scale.data(), zp.data(), 0, 0, 255) == REF_OK);
  for (int bits : {2, 8, 16, 24, 32})
    for (int sg = 0; sg <= 1; ++sg)
      REQUIRE(hago_ref_simquant_wrap(x.data(), y.data(), O, C, I, scale.data(), zp.data(), 1, bits, sg, -(1 << 24), 1 << 24) == REF_OK);
  REQUIRE(hago_ref_quantize(x.data(), q.data(), O, C, I, scale.data(), zp.data(), 1, i32min, i32max) == REF_OK);
  REQUIRE(hago_ref_dequantize(q.data(), y.data(), O, C, I, scale.data(), zp.data(), 1) == REF_OK);
  REQUIRE(hago_ref_absmax(x.data(), O, C, I, 1, thr.data()) == REF_OK);
  REQUIRE(hago_ref_absmax(x.data(), O, C, I, 0, thr.data()) == REF_OK);
  REQUIRE(hago_ref_absmax(x.data(), 0, C, I, 1, thr.data()) == REF_OK);

  // dense and conv: operand extremes, sums and biases that wrap, every accumulator width, padding
  const int64_t M = 5, N = 4, K = 37;
  std::vector<uint8_t> au(M * K);
  std::vector<int8_t> ai(M * K), w8(N * K);
  std::vector<int16_t> a16(M * K), w16(N * K);
  for (auto& v : au) v = (uint8_t)(rnd() % 4 == 0 ? 255 : rnd());
  for (auto& v : ai) v = (int8_t)(rnd() % 4 == 0 ? -128 : (int8_t)rnd());
  for (auto& v : w8) v = (int8_t)(rnd() % 4 == 0 ? -128 : (int8_t)rnd());
  for (auto& v : a16) v = (int16_t)(rnd() % 3 == 0 ? -32768 : (int16_t)rnd());
  for (auto& v : w16) v = (int16_t)(rnd() % 3 == 0 ? -32768 : (int16_t)rnd());
  std::vector<int32_t> bias = {i32max, i32min, 0, -1}, mult = {1 << 30, i32max, (1 << 30) + 12345, 1 << 30}, shift = {0, 31, 7, 1};
  ref_requant rq{mult.data(), shift.data(), 1, REF_I8, -3, -128, 127, REF_ROUND_UPWARD};
  ref_requant rq_u8{mult.data(), shift.data(), 0, REF_U8, 200, 0, 255, REF_ROUND_HALF_AWAY};
  ref_requant rq_shift{nullptr, shift.data(), 1, REF_I8, 0, -128, 127, REF_ROUND_UPWARD};
  std::vector<int32_t> o32(M * N);
  std::vector<int16_t> o16(M * N);
  std::vector<int8_t> o8(M * N);
  for (int32_t acc : {REF_I32, REF_I24}) {
    REQUIRE(hago_ref_qdense(au.data(), REF_U8, 255, w8.data(), bias.data(), M, N, K, acc, nullptr, o32.data()) == REF_OK);
    REQUIRE(hago_ref_qdense(ai.data(), REF_I8, -128, w8.data(), bias.data(), M, N, K, acc, &rq, o8.data()) == REF_OK);
    REQUIRE(hago_ref_qdense_x(a16.data(), REF_I16, -32768, w16.data(), REF_I16, bias.data(), M, N, K, acc, nullptr, o32.data()) == REF_OK);
    REQUIRE(hago_ref_qdense_x(a16.data(), REF_I16, 7, w16.data(), REF_I16, bias.data(), M, N, K, acc, &rq_shift, o8.data()) == REF_OK);
  }
  REQUIRE(hago_ref_qdense(au.data(), REF_U8, 0, w8.data(), nullptr, M, N, K, REF_I16, nullptr, o16.data()) == REF_OK);
  REQUIRE(hago_ref_qdense(au.data(), REF_U8, 0, w8.data(), nullptr, M, N, K, REF_I16, &rq_u8, o8.data()) == REF_OK);
  REQUIRE(hago_ref_qdense(au.data(), REF_U8, 0, w8.data(), nullptr, M, N, 0, REF_I32, nullptr, o32.data()) == REF_OK);
  REQUIRE(hago_ref_qdense(au.data(), REF_U8, 0, w8.data(), nullptr, 0, N, K, REF_I32, nullptr, o32.data()) == REF_OK);
  REQUIRE(hago_ref_qdense_x(a16.data(), REF_I16, 0, w16.data(), REF_I16, nullptr, M, N, K, REF_I16, nullptr, o16.data()) != REF_OK);
  REQUIRE(hago_ref_requantize(o32.data(), REF_I32, 1, N, M, &rq, o8.data()) == REF_OK);
  REQUIRE(hago_ref_requantize(o16.data(), REF_I16, M, N, 1, &rq_shift, o8.data()) == REF_OK);

  // conv geometries: stride, asymmetric padding larger than the kernel's reach, 1x1, depthwise, both layouts
  struct G { int64_t B, C, H, W, O; int32_t KH, KW, sh, sw, ph, pw, groups; };
  const G geoms[] = {{2, 3, 5, 6, 4, 3, 3, 1, 1, 1, 1, 1}, {1, 4, 7, 5, 4, 3, 2, 2, 3, 2, 0, 4}, {1, 2, 4, 4, 6, 1, 1, 1, 1, 0, 0, 1},
                     {1, 2, 3, 3, 2, 5, 5, 1, 1, 2, 2, 2}, {1, 6, 2, 9, 3, 2, 4, 1, 2, 3, 3, 1}};
  for (const G& g : geoms)
    for (int32_t layout : {REF_NCHW, REF_NHWC}) {
      const int64_t OH = (g.H + 2 * g.ph - g.KH) / g.sh + 1, OW = (g.W + 2 * g.pw - g.KW) / g.sw + 1;
      const int64_t na = g.B * g.C * g.H * g.W, nw = g.O * (g.C / g.groups) * g.KH * g.KW, no = g.B * g.O * OH * OW;
      std::vector<uint8_t> ca(na);
      std::vector<int8_t> cw(nw);
      std::vector<int16_t> ca16(na), cw16(nw);
      for (auto& v : ca) v = (uint8_t)rnd();
      for (auto& v : cw) v = (int8_t)rnd();
      for (auto& v : ca16) v = (int16_t)rnd();
      for (auto& v : cw16) v = (int16_t)rnd();
      std::vector<int32_t> cb(g.O, i32max), cm(g.O, i32max), cs(g.O, 13), co32(no);
      std::vector<int16_t> co16(no);
      std::vector<uint8_t> co8(no);
      ref_requant crq{cm.data(), cs.data(), 1, REF_U8, 128, 0, 255, REF_ROUND_UPWARD};
      REQUIRE(hago_ref_qconv2d(ca.data(), REF_U8, 128, cw.data(), cb.data(), layout, g.B, g.C, g.H, g.W, g.O, g.KH, g.KW, g.sh, g.sw,
                               g.ph, g.pw, g.groups, REF_I32, nullptr, co32.data()) == REF_OK);
      REQUIRE(hago_ref_qconv2d(ca.data(), REF_U8, 3, cw.data(), nullptr, layout, g.B, g.C, g.H, g.W, g.O, g.KH, g.KW, g.sh, g.sw,
                               g.ph, g.pw, g.groups, REF_I16, nullptr, co16.data()) == REF_OK);
      REQUIRE(hago_ref_qconv2d(ca.data(), REF_U8, 3, cw.data(), cb.data(), layout, g.B, g.C, g.H, g.W, g.O, g.KH, g.KW, g.sh, g.sw,
                               g.ph, g.pw, g.groups, REF_I24, &crq, co8.data()) == REF_OK);
      REQUIRE(hago_ref_qconv2d_x(ca16.data(), REF_I16, -5, cw16.data(), REF_I16, cb.data(), layout, g.B, g.C, g.H, g.W, g.O, g.KH,
                                 g.KW, g.sh, g.sw, g.ph, g.pw, g.groups, REF_I32, nullptr, co32.data()) == REF_OK);
    }
  std::puts("oracle sanitizer driver: ok");
  return 0;
}
