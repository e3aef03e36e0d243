// Host-sanitizer driver (test infrastructure, CPU only): the C oracle and the CPU build of the HIP library's
// device bit logic, both compiled with -fsanitize=address,undefined into this one program, run over a reduced
// pin set -- every top-13-bit binary32 pattern with zero and all-ones fillers, every 16-bit source pattern,
// random patterns, ragged and empty arrays -- and compared with each other element by element.
// Prints "sanitize OK ..." and returns 0 when nothing differs; any sanitizer report aborts the run.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

extern "C" {
// oracle/hif8_oracle.c
double hif8o_decode_value(uint8_t code);
uint8_t hif8o_encode_one_t(float y, uint32_t mode, int src_kind, uint32_t t32);
uint32_t hif8o_sr_threshold(uint64_t seed, uint64_t index);
void hif8o_set_sr_seed(uint64_t seed);
void hif8o_set_sr_index_base(uint64_t base);
void hif8o_encode_f32(const float* src, uint8_t* dst, size_t n, float scale, uint32_t mode);
void hif8o_encode_bf16(const uint16_t* src, uint8_t* dst, size_t n, float scale, uint32_t mode);
void hif8o_encode_f16(const uint16_t* src, uint8_t* dst, size_t n, float scale, uint32_t mode);
void hif8o_decode_f32(const uint8_t* src, float* dst, size_t n, float scale);
void hif8o_decode_bf16(const uint8_t* src, uint16_t* dst, size_t n, float scale);
void hif8o_fake_quant_bf16(const uint16_t* src, uint16_t* dst, uint8_t* codes, size_t n, float scale, uint32_t mode);
float hif8o_amax_f32(const float* src, size_t n);
float hif8o_amax_bf16(const uint16_t* src, size_t n);
float hif8o_amax_f16(const uint16_t* src, size_t n);
float hif8o_scale_from_amax(float amax, float target, int pow2);
void hif8o_scale_sweep(const void* x, size_t n, int src_kind, int e_lo, int count, uint32_t mode, double* err);
void hif8o_amax_axis(const void* x, size_t rows, size_t cols, int src_kind, int axis, float* amax_out);
// tests/devfn_host/devfn_host.cpp
void devfn_encode_bits(const uint32_t*, uint8_t*, size_t, uint32_t, int, uint64_t);
void devfn_encode_bits_hr_table(const uint32_t*, uint8_t*, size_t, uint32_t);
void devfn_encode_bits_hr16_stream(const uint32_t*, uint8_t*, size_t, uint32_t, int);
void devfn_encode_bits_sr_table(const uint32_t*, uint8_t*, size_t, uint32_t, uint64_t);
void devfn_decode_bits(const uint8_t*, uint32_t*, size_t);
void devfn_narrow_bf16(const uint32_t*, uint16_t*, size_t);
void devfn_scale_from_amax(const float*, float*, size_t, float, int);
uint32_t devfn_ragged_round_split(size_t, size_t, size_t);
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t next_u64() {  // xorshift64*: any deterministic filler will do
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return rng_state * 0x2545F4914F6CDD1Dull;
}
static float as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t as_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

int main() {
  size_t bad = 0, checked = 0;
  // binary32 patterns: every top-13-bit pattern with zero / all-ones / random low bits, plus random patterns;
  // NaNs are made quiet, as the scale multiply of the kernels returns them
  std::vector<uint32_t> y;
  for (uint32_t i = 0; i < 8192; ++i) {
    y.push_back(i << 19); y.push_back((i << 19) | 0x7FFFFu); y.push_back((i << 19) | ((uint32_t)next_u64() & 0x7FFFFu));
  }
  for (int i = 0; i < 200000; ++i) y.push_back((uint32_t)next_u64());
  for (auto& v : y) if ((v & 0x7F800000u) == 0x7F800000u && (v & 0x7FFFFFu)) v |= 0x400000u;
  const size_t n = y.size();
  std::vector<uint8_t> c_dev(n), c_dev2(n), c_orc(n);
  const uint64_t seed = 0x1234567890ABCDEFull;
  for (uint32_t mode : {0u, 1u, 2u, 3u, 4u, 0x10u, 0x21u, 0x34u}) {
    for (int srck = 0; srck < 3; ++srck) {
      devfn_encode_bits(y.data(), c_dev.data(), n, mode, srck, seed);
      for (size_t i = 0; i < n; ++i)
        c_orc[i] = hif8o_encode_one_t(as_float(y[i]), mode, srck, hif8o_sr_threshold(seed, i));
      for (size_t i = 0; i < n; ++i) { bad += c_dev[i] != c_orc[i]; ++checked; }
      if ((mode & 15) == 1 || (mode & 15) == 3) {
        if (srck == 0) devfn_encode_bits_hr_table(y.data(), c_dev2.data(), n, mode);
        else devfn_encode_bits_hr16_stream(y.data(), c_dev2.data(), n, mode, srck);
        for (size_t i = 0; i < n; ++i) bad += c_dev[i] != c_dev2[i];
      }
      if ((mode & 15) == 4 && srck == 0) {
        devfn_encode_bits_sr_table(y.data(), c_dev2.data(), n, mode, seed);
        for (size_t i = 0; i < n; ++i) bad += c_dev[i] != c_dev2[i];
      }
    }
  }
  // decode: all 256 codes, oracle value against the device pattern
  std::vector<uint8_t> codes(256);
  std::vector<uint32_t> dbits(256);
  for (int i = 0; i < 256; ++i) codes[i] = (uint8_t)i;
  devfn_decode_bits(codes.data(), dbits.data(), 256);
  for (int i = 0; i < 256; ++i) {
    const double v = hif8o_decode_value((uint8_t)i);
    const float f = as_float(dbits[i]);
    if (v != v) bad += !(f != f); else bad += (double)f != v;
    ++checked;
  }
  // the oracle's array entry points on empty, tiny and ragged arrays (bounds), every 16-bit pattern included
  std::vector<uint16_t> h16(65536 + 3);
  for (size_t i = 0; i < h16.size(); ++i) h16[i] = (uint16_t)i;
  std::vector<float> xf(n);
  for (size_t i = 0; i < n; ++i) xf[i] = as_float(y[i]);
  for (size_t m : {(size_t)0, (size_t)1, (size_t)7, (size_t)4099, h16.size()}) {
    std::vector<uint8_t> c(m + 1, 0xA5);
    std::vector<uint16_t> o16(m + 1, 0xA5A5);
    std::vector<float> o32(m + 1);
    hif8o_set_sr_seed(seed); hif8o_set_sr_index_base(((uint64_t)1 << 32) - 2);
    hif8o_encode_bf16(h16.data(), c.data(), m, 0.37f, 4u | 0x10u);
    hif8o_encode_f16(h16.data(), c.data(), m, 3.0f, 1u);
    hif8o_encode_f32(xf.data(), c.data(), m, 1.0f, 3u);
    hif8o_set_sr_seed(0); hif8o_set_sr_index_base(0);
    hif8o_fake_quant_bf16(h16.data(), o16.data(), c.data(), m, 4.0f, 0u);
    hif8o_decode_bf16(c.data(), o16.data(), m, 4.0f);
    hif8o_decode_f32(c.data(), o32.data(), m, 0.5f);
    bad += c[m] != 0xA5 || o16[m] != 0xA5A5;   // nothing written past the end
    (void)hif8o_amax_bf16(h16.data(), m); (void)hif8o_amax_f16(h16.data(), m); (void)hif8o_amax_f32(xf.data(), m);
    double err[16];
    hif8o_scale_sweep(xf.data(), m, 0, -4, 10, 0u, err);
    if (m >= 12) {
      std::vector<float> am(m);
      hif8o_amax_axis(h16.data(), 3, m / 3, 1, 0, am.data());
      hif8o_amax_axis(h16.data(), 3, m / 3, 1, 1, am.data());
    }
  }
  // scale from amax: device arithmetic against the oracle on every pattern of the list
  std::vector<float> s(n);
  for (int pow2 = 0; pow2 < 2; ++pow2) {
    for (float target : {32768.0f, 1.0f, 3.0e38f}) {
      devfn_scale_from_amax(xf.data(), s.data(), n, target, pow2);
      for (size_t i = 0; i < n; ++i) {
        if (y[i] >> 31) continue;  // amax is a magnitude
        bad += as_bits(s[i]) != as_bits(hif8o_scale_from_amax(xf[i], target, pow2));
        ++checked;
      }
    }
  }
  std::vector<uint16_t> nb(n);
  devfn_narrow_bf16(y.data(), nb.data(), n);
  uint64_t acc = 0;
  for (int i = 0; i < 20000; ++i) acc += devfn_ragged_round_split(next_u64() % 100000 + 1, next_u64() % 100000 + 1, next_u64() % 400);
  printf("sanitize %s: %zu comparisons, %zu mismatches (%llu)\n", bad ? "FAILED" : "OK", checked, bad, (unsigned long long)acc);
  return bad != 0;
}
