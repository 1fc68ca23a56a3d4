// Test infrastructure: replays cases from stdin through the library's host functions (draft_host.cpp),
// built with -fsanitize=address,undefined; tests/test_host_sanitizers.py generates the cases and
// compares what this prints with the oracle.  One case per line:
//   chk B parent[B]                                         -> status
//   plan n_seq seq[n_seq] n_lens lens[n_lens] max_spine anchor V K ids[V*K] scores[V*K] B p_hat rho D thr bypass
//                                                           -> status mode n tokens[n] parent[n] is_spine[n]
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "goose.h"

int main() {
  std::string op;
  while (std::cin >> op) {
    if (op == "chk") {
      int B;
      std::cin >> B;
      std::vector<int32_t> p(B > 0 ? B : 0);
      for (auto& v : p) std::cin >> v;
      std::printf("%d\n", goose_check_parent(p.empty() ? nullptr : p.data(), B));
    } else if (op == "plan") {
      int n_seq, n_lens, max_spine, anchor, V, K, B, D, bypass;
      double p_hat, rho, thr;
      std::cin >> n_seq;
      std::vector<int32_t> seq(n_seq);
      for (auto& v : seq) std::cin >> v;
      std::cin >> n_lens;
      std::vector<int32_t> lens(n_lens);
      for (auto& v : lens) std::cin >> v;
      std::cin >> max_spine >> anchor >> V >> K;
      std::vector<int32_t> ids((size_t)V * K);
      std::vector<float> sc((size_t)V * K);
      for (auto& v : ids) std::cin >> v;
      for (auto& v : sc) std::cin >> v;
      std::cin >> B >> p_hat >> rho >> D >> thr >> bypass;
      // exactly B elements: an overrun of the outputs is the sanitizer's to catch
      std::vector<int32_t> tok(B), par(B);
      std::vector<uint8_t> spn(B);
      int32_t n = 0, mode = -1;
      const int rc = goose_plan_cycle(seq.data(), n_seq, lens.data(), n_lens, max_spine, anchor, ids.data(), sc.data(), V, K,
                                      B, p_hat, rho, D, thr, bypass, tok.data(), par.data(), spn.data(), &n, &mode);
      std::printf("%d %d %d", rc, mode, n);
      for (int i = 0; i < n; ++i) std::printf(" %d", tok[i]);
      for (int i = 0; i < n; ++i) std::printf(" %d", par[i]);
      for (int i = 0; i < n; ++i) std::printf(" %d", (int)spn[i]);
      std::printf("\n");
    } else {
      std::fprintf(stderr, "unknown op %s\n", op.c_str());
      return 2;
    }
  }
  return 0;
}
