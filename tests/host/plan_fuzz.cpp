// host-only fuzz of the planning entry points under ASan/UBSan (no device needed)
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>
#include <random>
#include "onebitlamb.h"
int main() {
  std::mt19937_64 rng(12345);
  const int64_t kinds[] = {0, 1, 2, 3, 255, 256, 1023, 1024, 1025, 4096, 8191, 8192, 8193, 16384, 24576, 40000, 65536,
                           100000, 63 * 8192, 64 * 8192, 64 * 8192 + 5000, 70 * 8192 + 1, 100 * 8192};
  const int nk = sizeof(kinds) / sizeof(kinds[0]);
  const int Ws[] = {1, 2, 3, 4, 5, 8, 16, 64, 255};
  const int64_t mts[] = {0, 1, 2, 3, 5, 66, 1000};
  long checks = 0;
  for (int it = 0; it < 400; ++it) {
    const int L = 1 + (int)(rng() % 16);
    std::vector<int64_t> off(L + 1, 0);
    for (int l = 0; l < L; ++l) off[l + 1] = off[l] + kinds[rng() % nk];
    if (off[L] == 0) off[L] = 1 + (int64_t)(rng() % 5000);
    const int W = Ws[rng() % 9];
    const int64_t mt = mts[rng() % 7];
    ob_lamb_config cfg{};
    cfg.num_layers = L; cfg.layer_offsets = off.data(); cfg.num_workers = W; cfg.server_chunk = 0;
    cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.beta3 = 0.9f; cfg.eta = 1e-6f; cfg.c_min = 0.01f; cfg.c_max = 0.3f;
    cfg.r_min = 0.5f; cfg.r_max = 4.0f; cfg.r_threshold = 0.1f; cfg.weight_decay = 0.0f;
    const int64_t n_pad = ob_lamb_padded_len_for(off[L], W);
    const int64_t n_c = n_pad / W;
    const size_t spans = (size_t)W * (size_t)((n_c + 1023) / 1024);
    // exact-size heap buffers: any write past the end is caught
    std::vector<uint8_t> owner(spans), big(spans);
    std::vector<int32_t> listed(L);
    if (ob_lamb_plan_split(&cfg, mt, owner.data(), listed.data()) != OB_OK) { printf("plan_split failed it=%d\n", it); return 1; }
    if (ob_lamb_plan_big_tiles(&cfg, mt, big.data()) != OB_OK) { printf("plan_big failed it=%d\n", it); return 1; }
    for (size_t i = 0; i < spans; ++i) {
      if (owner[i] > 2 || big[i] > 1 || (big[i] && owner[i] != 1)) { printf("bad value it=%d\n", it); return 1; }
      ++checks;
    }
  }
  // the static entry's argument checks and the null-context paths touch no device either
  ob_lamb_state st{};
  if (ob_lamb_compress_local(nullptr, &st, nullptr, nullptr, nullptr, nullptr) != OB_ERR_NULL) return 2;
  printf("ok %ld spans checked\n", checks);
  return 0;
}
