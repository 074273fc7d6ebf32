// Random call sequences, many of them invalid, on host-only contexts (no kernel is launched, no device memory is
// touched): built with AddressSanitizer and UBSan by tests/test_host_sanitized.py, so that an out-of-range index
// or an overflow in the bookkeeping of the C ABI's host side aborts the run.  The results are not checked here
// (tests/test_abi.py compares them with the oracle); only memory safety and defined behaviour are.
#include "recover.h"
#include <stdio.h>
#include <stdlib.h>
#include <vector>
static unsigned long long s = 88172645463325252ull;
static unsigned rnd() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return (unsigned)(s >> 11); }
int main() {
  long calls = 0, oks = 0;
  for (int trial = 0; trial < 400; ++trial) {
    const int W = 1 + rnd() % 64, G = 1 + rnd() % 4, T = 1 + rnd() % 9;
    std::vector<int64_t> off(T + 1, 0);
    for (int t = 0; t < T; ++t) off[t + 1] = off[t] + (rnd() % 5 == 0 ? 0 : rnd() % 1000);
    std::vector<float *> snap(W, nullptr);
    recover_config cfg = {};
    cfg.W_init = W; cfg.G_init = G; cfg.n_elems = off[T]; cfg.n_tensors = T; cfg.tensor_offsets = off.data();
    cfg.snap = (rnd() & 1) ? snap.data() : nullptr;
    cfg.flags = RECOVER_FLAG_HOST_ONLY | ((rnd() & 3) == 0 ? RECOVER_FLAG_ADAPTIVE : 0) | ((rnd() & 3) == 0 ? RECOVER_FLAG_ANY_ORDER : 0);
    recover_ctx *c = nullptr;
    if (recover_init(&cfg, &c) != RECOVER_OK) { printf("init failed: %s\n", recover_last_error(nullptr)); return 1; }
    std::vector<int32_t> role(W), target(W), contributed(W), bm(W);
    std::vector<uint32_t> ids(64);
    unsigned next_id = 0;
    for (int step = 0; step < 600; ++step) {
      int rc = 0;
      const int r = (int)(rnd() % (W + 2)) - 1, tb = rnd() % (T + 1), te = rnd() % (T + 2);
      switch (rnd() % 12) {
        case 0: case 1: case 2: case 3: rc = recover_accumulate(c, r, next_id++, nullptr, rnd() % 3, (rnd() & 3) ? 0 : tb, (rnd() & 3) ? T : te, nullptr); break;
        case 4: rc = recover_accumulate_snapshot(c, r, next_id++, nullptr, RECOVER_F32, 0, T, nullptr); break;
        case 5: rc = recover_snapshot(c, r, tb, te, nullptr); break;
        case 6: rc = recover_restore(c, r, rnd() & 1, nullptr); break;
        case 7: {
          int32_t f[4]; int n = rnd() % 4;
          for (int k = 0; k < n; ++k) f[k] = (int)(rnd() % (W + 1)) - (rnd() % 16 == 0);
          recover_decision d = {}; d.role = role.data(); d.target = target.data(); d.contributed = contributed.data(); d.is_boundary_minor = bm.data();
          rc = recover_policy_adjust(c, f, (rnd() % 8 == 0) ? 0 : n, &d);
          break;
        }
        case 8: rc = recover_reduce(c, (rnd() & 1) ? 0 : tb, (rnd() & 1) ? T : te, rnd() % 3 == 0 ? RECOVER_REDUCE_INPLACE : 0, nullptr); break;
        case 9: rc = (rnd() & 1) ? recover_adamw_step(c, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.1f, nullptr)
                               : recover_reduce_adamw_step(c, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.1f, rnd() & 1, nullptr); break;
        case 10: { recover_decision d = {}; d.role = role.data(); d.target = target.data(); rc = recover_query(c, &d); break; }
        case 11: rc = recover_committed_ids(c, r, ids.data(), rnd() % 65); break;
      }
      ++calls; oks += rc >= 0;
      if (rnd() % 50 == 0) { std::vector<int32_t> rep(W); std::vector<uint32_t> mb(W); for (int k = 0; k < W; ++k) { rep[k] = rnd() % W; mb[k] = next_id++; }
        std::vector<int32_t> st(W); (void)recover_accumulate_many(c, 1 + rnd() % W, rep.data(), mb.data(), nullptr, RECOVER_F32, st.data(), nullptr); }
    }
    (void)recover_adamw_step_static(c, (int)(rnd() % 70) - 3, rnd() & 1, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.1f, nullptr);
    recover_destroy(c);
  }
  printf("fuzz ok: %ld calls, %ld accepted\n", calls, oks);
  return 0;
}
