// Calls the host half of the library -- roast_tile_index and the argument validation that every entry
// point runs before it launches anything -- so that a build of csrc/roast_api.hip with host-side
// -fsanitize=address,undefined reports out-of-bounds accesses or undefined integer operations.  No call
// here reaches a kernel launch: each one is refused by validation, sized zero, or host-only.
#include <stdio.h>

#include <vector>

#include "roast.h"

int main() {
  const uint64_t primes[4] = {2, 65537, 2147483647ull, 4294967291ull};
  int bad = 0;
  for (uint64_t P : primes)
    for (uint32_t align = 1; align <= 4; align += 3) {
      roast_hash h{P, 5 % P, 7 % P, 11 % P, 13 % P, 17 % P, 19 % P, 23 % P, 29 % P, 1, align};
      for (int Z1 = 1; Z1 <= 9; Z1 += 2)
        for (int Z2 = 1; Z2 <= 9; Z2 += 4)
          for (int H = 1; H < 40; H += 13)
            for (int O = 1; O < 40; O += 19) {
              const int64_t L = (int64_t)Z1 * Z2;
              for (int64_t m : {L, L + 1, L + 1000}) {
                roast_mm_desc d{H, O, Z1, Z2, m, 0xffffffffu, 1.f, h};
                const int64_t ntx = (H + Z1 - 1) / Z1, nty = (O + Z2 - 1) / Z2;
                std::vector<int64_t> off(ntx * nty);
                std::vector<int8_t> sg(ntx * nty);
                if (roast_tile_index(&d, off.data(), sg.data()) != ROAST_OK) ++bad;
                for (auto o : off) bad += (o < 0 || o > m - L || o % align != 0);
                for (auto s : sg) bad += (s != 1 && s != -1);
                if (roast_tile_index(&d, nullptr, sg.data()) != ROAST_OK) ++bad;
              }
            }
    }
  roast_hash h{2147483647ull, 5, 7, 11, 13, 17, 19, 23, 29, 1, 1};
  float x = 0.f;
  int64_t row = 0;
  uint32_t tab = 0;
  {  // refused before any launch
    roast_mm_desc d{8, 8, 4, 4, 8, 0u, 1.f, h};
    bad += roast_tile_index(&d, nullptr, nullptr) != ROAST_ERR_RANGE;                 // |M| < Z1*Z2
    d.m_size = 64;
    bad += roast_mm_fwd(&d, ROAST_F32, -1, &x, 8, &x, nullptr, &x, 8, nullptr) != ROAST_ERR_ARG;
    bad += roast_mm_fwd(&d, ROAST_F32, 4, &x, 7, &x, nullptr, &x, 8, nullptr) != ROAST_ERR_ARG;       // ld too small
    bad += roast_mm_fwd(&d, ROAST_F32, 0, nullptr, 8, nullptr, nullptr, nullptr, 8, nullptr) != ROAST_OK;   // I == 0
    // (enum arguments outside their declared values are exercised through ctypes in
    // tests/test_library_host.py: forming such a value in C++ is itself undefined behaviour)
    bad += roast_mm_bwd_dM(&d, ROAST_F32, 4, &x, 8, &x, 8, &x, ROAST_REDUCE_DETERMINISTIC, nullptr, 0, nullptr) != ROAST_ERR_WORKSPACE;
    d.Z1 = 0;
    bad += roast_mm_fwd(&d, ROAST_F32, 4, &x, 8, &x, nullptr, &x, 8, nullptr) != ROAST_ERR_SHAPE;
    d.Z1 = 4; d.hash.a0 = d.hash.P;
    bad += roast_mm_fwd(&d, ROAST_F32, 4, &x, 8, &x, nullptr, &x, 8, nullptr) != ROAST_ERR_RANGE;
    bad += roast_mm_bwd_dM_workspace(&d, 4, ROAST_REDUCE_DETERMINISTIC) != 0;
  }
  {
    roast_embed_desc e{16, 4, 3, 1.f, h};
    bad += roast_embed_fwd(&e, 1, &row, &tab, &x, &x, nullptr) != ROAST_ERR_RANGE;    // |M| < Z
    e.m_size = 100;
    bad += roast_embed_fwd(&e, 1, nullptr, &tab, &x, &x, nullptr) != ROAST_ERR_ARG;
    bad += roast_embed_fwd(&e, 0, nullptr, nullptr, nullptr, nullptr, nullptr) != ROAST_OK;
    bad += roast_embed_bwd(&e, 1, &row, &tab, &x, &x, ROAST_REDUCE_DETERMINISTIC, nullptr, 0, nullptr) != ROAST_ERR_WORKSPACE;
    bad += roast_embed_bwd_workspace(&e, 1 << 20, ROAST_REDUCE_ATOMIC) == 0;
    bad += roast_embed_bwd_workspace(&e, 1 << 20, ROAST_REDUCE_DETERMINISTIC) == 0;
    bad += roast_embed_bag_fwd(&e, 4, -1, &row, &tab, &row, &x, &x, nullptr) != ROAST_ERR_ARG;
  }
  {
    roast_optim_desc o{ROAST_OPT_ADAM, 1e-3f, 0.f, 0.9f, 0.999f, 1e-8f, 0, 1};
    bad += roast_optim_step(&o, 16, &x, &x, &x, &x, nullptr, nullptr) != ROAST_ERR_ARG;   // step < 1
    bad += roast_m_shadow_bytes(47185) < 2 * 2 * 47185;
    bad += roast_m_planes_bytes(47185) < 3 * roast_m_shadow_bytes(47185);
    bad += roast_m_shadow_bf16(&x, -1, &x, nullptr) != ROAST_ERR_ARG;
  }
  for (int s = 0; s <= 7; ++s) bad += roast_status_string((roast_status)s) == nullptr;
  printf("host api sanitizer driver: %d failures\n", bad);
  return bad != 0;
}
