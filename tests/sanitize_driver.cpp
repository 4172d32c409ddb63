// Host-only exercise of the encoder and the validator under ASan/UBSan: random matrices, every option, carried
// dictionaries, and corrupted containers.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>
#include "../include/tq.h"
int main() {
  std::mt19937 rng(7);
  int n_ok = 0, n_bad = 0;
  for (int it = 0; it < 300; ++it) {
    const uint32_t rows = 1 + rng() % 70, cols = 2 * (1 + rng() % 400);
    std::vector<float> w((size_t)rows * cols);
    std::normal_distribution<float> nd(0.f, 0.02f);
    const bool sparse = rng() % 3 == 0;
    for (auto& v : w) v = (sparse && rng() % 10) ? 0.f : nd(rng);
    tq_encode_opts o;
    std::memset(&o, 0, sizeof o);
    o.lmax = 1 + rng() % 4;
    const uint32_t segs[] = {16, 32, 64, 96, 128, 256, 1024};
    o.seg_cols = segs[rng() % 7];
    o.max_entries = (rng() % 2) ? 0 : 256 + rng() % 3000;
    o.bits = (rng() % 2) ? 0 : 2 + rng() % 7;
    o.packing = (o.bits >= 2 && o.bits <= 4 && rng() % 2) ? 1 : 0;
    o.dictionary = (o.lmax <= 2 && rng() % 3 == 0) ? 1 : 0;
    o.n_threads = 1 + rng() % 4;
    void* blob = nullptr;
    size_t bytes = 0;
    int rc = tq_encode(w.data(), rows, cols, &o, &blob, &bytes);
    if (rc != TQ_OK) { std::printf("encode rc %d: %s\n", rc, tq_last_error_string()); return 1; }
    tq_info info;
    if (tq_validate_blob(blob, bytes, &info) != TQ_OK) { std::printf("validate: %s\n", tq_last_error_string()); return 1; }
    ++n_ok;
    // a second matrix that goes on from the first one's dictionary
    void* blob2 = nullptr;
    size_t bytes2 = 0;
    tq_encode_opts o2 = o;
    o2.dict_from = blob;
    o2.dict_from_bytes = bytes;
    rc = tq_encode(w.data(), rows, cols, &o2, &blob2, &bytes2);
    if (rc != TQ_OK) { std::printf("encode (carried) rc %d: %s\n", rc, tq_last_error_string()); return 1; }
    if (tq_validate_blob(blob2, bytes2, nullptr) != TQ_OK) { std::printf("validate (carried): %s\n", tq_last_error_string()); return 1; }
    tq_free_blob(blob2);
    // corrupt a few bytes and truncate: validation must answer, never crash
    for (int k = 0; k < 20; ++k) {
      std::vector<uint8_t> bad((uint8_t*)blob, (uint8_t*)blob + bytes);
      const int flips = 1 + rng() % 4;
      for (int f = 0; f < flips; ++f) bad[rng() % (k % 2 ? 256 : bad.size())] ^= (uint8_t)(1u << (rng() % 8));
      size_t nb = (k % 5 == 0) ? rng() % bad.size() : bad.size();
      if (tq_validate_blob(bad.data(), nb, nullptr) != TQ_OK) ++n_bad;
    }
    tq_free_blob(blob);
  }
  std::printf("%d containers encoded and validated, %d corrupted ones refused\n", n_ok, n_bad);
  return 0;
}
