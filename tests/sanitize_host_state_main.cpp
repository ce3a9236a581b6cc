// Sanitizer driver for the library's host-side state (test helper, CPU only): built by tests/test_oracle_sanitizers.py
// together with csrc/host_state.hip (plain C++, no device code) under -fsanitize=address,undefined and run once.
// It drives the pager through a seeded random schedule of reserve / trim / end-of-session calls with a shadow model
// (every page owned by at most one session, free + owned = all pages, nothing taken on a refused call), and the
// stride policy over a grid including its refusals.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <set>
#include <vector>

#include "../paper_2601_00644_amd/csrc/host_state.hip"

static uint64_t rng = 12345;
static uint32_t next_u32() {
  rng = rng * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng >> 33);
}

int main() {
  const int NP = 97, NS = 7, MPS = 23;
  fsv_pager *p = nullptr;
  if (fsv_pager_create(NP, NS, MPS, &p) != FSV_OK || !p) return 1;
  fsv_pager_destroy(p);
  if (fsv_pager_create(0, NS, MPS, &p) != FSV_E_INVALID_ARG || p != nullptr) return 2;
  if (fsv_pager_create(NP, NS, MPS, &p) != FSV_OK) return 3;
  std::vector<std::vector<int32_t>> shadow(NS);
  std::vector<int32_t> row(MPS + 4, -7);
  for (int step = 0; step < 20000; ++step) {
    const int s = (int)(next_u32() % (NS + 2)) - 1;   // -1 and NS are refused
    const int n = (int)(next_u32() % (16 * MPS + 40)) - 8;
    const int before_free = fsv_pager_free_pages(p);
    if (next_u32() % 3) {
      const int rc = fsv_pager_reserve(p, s, n, (next_u32() & 1) ? row.data() : nullptr);
      const bool bad = s < 0 || s >= NS || n < 0;
      if (bad) { if (rc != FSV_E_INVALID_ARG || fsv_pager_free_pages(p) != before_free) return 10; continue; }
      const int need = (n + 15) / 16, have = (int)shadow[s].size();
      if (need > MPS || need - have > before_free) {
        if (rc != FSV_E_CAPACITY || fsv_pager_free_pages(p) != before_free || fsv_pager_session_pages(p, s) != have) return 11;
        continue;
      }
      if (rc != FSV_OK) return 12;
      if (fsv_pager_session_pages(p, s) != (need > have ? need : have)) return 13;
      std::vector<int32_t> full(MPS + 4, -7);
      if (fsv_pager_reserve(p, s, 0, full.data()) != FSV_OK) return 14;   // asks for nothing more: reports what it owns
      shadow[s].assign(full.begin(), full.begin() + fsv_pager_session_pages(p, s));
      if (full[shadow[s].size()] != -7) return 15;                          // nothing written past the owned pages
    } else {
      const int rc = fsv_pager_trim(p, s, n);
      const bool bad = s < 0 || s >= NS || n < 0;
      if (bad) { if (rc != FSV_E_INVALID_ARG) return 20; continue; }
      const int keep = (n + 15) / 16, have = (int)shadow[s].size(), rel = have > keep ? have - keep : 0;
      if (rc != rel) return 21;
      shadow[s].resize(have - rel);
    }
    std::set<int32_t> seen;
    size_t owned = 0;
    for (auto &v : shadow) { owned += v.size(); for (int32_t g : v) { if (g < 0 || g >= NP || !seen.insert(g).second) return 30; } }
    if ((int)owned + fsv_pager_free_pages(p) != NP) return 31;
  }
  fsv_pager_destroy(p);
  fsv_pager_destroy(nullptr);

  fsv_latency_model m{};
  m.alpha_edge = 0.012; m.beta = 0.002; m.bits_per_token = 17; m.header_bits = 320; m.t_prop = 0.02; m.t_base = 0.006;
  m.delta_cloud = 0.0002; m.t_down = 0.005;
  double acc = 0.0;
  for (int model = 0; model < 2; ++model)
    for (double rate = 1e2; rate < 1e9; rate *= 7.3)
      for (double g = 0.0; g <= 1.0; g += 0.125)
        for (int kmax = 1; kmax <= 33; kmax += 8) {
          double obj = -1.0;
          const int k = fsv_policy_stride(&m, rate, g, kmax, model, &obj);
          if (k < 1 || k > kmax || !(obj > 0.0)) return 40;
          const double t = fsv_policy_step_time(&m, rate, k, -1.0);
          if (!(t > 0.0) || !isfinite(t)) return 41;
          acc += k + fsv_policy_ema(g, k / 2, k, 0.1);
        }
  if (fsv_policy_stride(nullptr, 1e6, 0.5, 8, 0, nullptr) != FSV_E_INVALID_ARG || fsv_policy_stride(&m, 0.0, 0.5, 8, 0, nullptr) != FSV_E_INVALID_ARG ||
      fsv_policy_stride(&m, 1e6, 0.5, 0, 0, nullptr) != FSV_E_INVALID_ARG || fsv_policy_stride(&m, 1e6, 0.5, 8, 2, nullptr) != FSV_E_INVALID_ARG ||
      fsv_policy_stride(&m, 1e6, NAN, 8, 0, nullptr) != FSV_E_INVALID_ARG)
    return 42;
  if (fsv_policy_step_time(&m, -1.0, 3, -1.0) != -1.0 || fsv_policy_ema(0.7, 3, 0, 0.1) != 0.7) return 43;
  printf("ok %.3f\n", acc);
  return 0;
}
