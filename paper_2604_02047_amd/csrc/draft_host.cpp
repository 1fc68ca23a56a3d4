// Host side of a decoding cycle: validation of a parent array, context n-gram match, budget split, spine-tree construction,
// spine-ratio tiers and their moving average (Sec. 4.1, Sec. 4.3, Alg. BuildSpineTree, Alg.
// "Decoding Loop" and the note on ContextMatch below it; hyperparameter table of App. C).
// Plain C++ on host memory: per cycle this is a few microseconds on ~100 tokens, next to a
// multi-millisecond verification pass; the successor tables are a host mirror of the rows the
// harvest kernel wrote (the caller copies the B touched rows back with the cycle's results).
#include <cmath>
#include <cstdint>
#include <vector>

#include "goose.h"

extern "C" {

int goose_check_parent(const int32_t* h_parent, int B) {
  if (!h_parent || B < 1 || B > GOOSE_MAX_B) return GOOSE_ERR_ARG;
  if (h_parent[0] != -1) return GOOSE_ERR_NOT_TOPOLOGICAL;
  for (int i = 1; i < B; ++i)
    if (h_parent[i] < 0 || h_parent[i] >= i) return GOOSE_ERR_NOT_TOPOLOGICAL;
  return GOOSE_OK;
}

int goose_context_match(const int32_t* h_seq, int n_seq, const int32_t* h_lens, int n_lens, int max_len,
                        int32_t* h_draft, int32_t* h_m, int32_t* h_consensus) {
  if (!h_seq || !h_lens || !h_draft || !h_m || !h_consensus || n_seq < 0 || n_lens < 1 || n_lens > 8 || max_len < 1)
    return GOOSE_ERR_ARG;
  *h_m = 0;
  *h_consensus = 0;
  int best_n = 0, best_at = -1;        // match of the largest n: continuation starts at best_at
  int firsts[8];
  int n_found = 0;
  for (int q = 0; q < n_lens; ++q) {
    const int n = h_lens[q];
    if (n < 1) return GOOSE_ERR_ARG;
    if (n_seq < n + 1) continue;
    const int32_t* tail = h_seq + n_seq - n;
    for (int j = n_seq - n - 1; j >= 0; --j) {  // most recent earlier occurrence
      bool same = true;
      for (int e = 0; e < n && same; ++e) same = h_seq[j + e] == tail[e];
      if (!same) continue;
      // j + n <= n_seq - 1: at least one token follows the match
      firsts[n_found++] = h_seq[j + n];
      if (n > best_n) { best_n = n; best_at = j + n; }
      break;
    }
  }
  if (n_found == 0) return GOOSE_OK;
  for (int a = 0; a < n_found; ++a)
    for (int b = a + 1; b < n_found; ++b)
      if (firsts[a] == firsts[b]) *h_consensus = 1;
  int m = n_seq - best_at;
  if (m > max_len) m = max_len;
  for (int e = 0; e < m; ++e) h_draft[e] = h_seq[best_at + e];
  *h_m = m;
  return GOOSE_OK;
}

int goose_spine_budget(int B, int m, double r, double rho, int32_t* b_s, int32_t* b_r, int32_t* b_rho) {
  if (!b_s || !b_r || !b_rho || B < 1 || m < 0 || !(r > 0.0 && r < 1.0) || !(rho > 0.0 && rho < 1.0))
    return GOOSE_ERR_ARG;
  int s = (int)std::floor((double)B * r);
  if (m < s) s = m;
  if (s > B - 1) s = B - 1;
  const int root = (int)std::floor((double)(B - 1 - s) * (1.0 - rho));
  *b_s = s;
  *b_r = root;
  *b_rho = B - 1 - s - root;
  return GOOSE_OK;
}

int goose_build_spine_tree(int32_t anchor, const int32_t* h_draft, int m, const int32_t* h_succ_ids,
                           const float* h_succ_scores, int vocab, int K, int B, double r, double rho, int D,
                           double min_score, int32_t* h_tokens, int32_t* h_parent, uint8_t* h_is_spine,
                           int32_t* h_n) {
  if (!h_succ_ids || !h_succ_scores || !h_tokens || !h_parent || !h_is_spine || !h_n || (m > 0 && !h_draft))
    return GOOSE_ERR_ARG;
  if (B < 1 || B > GOOSE_MAX_B || K < 1 || vocab < 1 || D < 0 || m < 0) return GOOSE_ERR_ARG;
  int32_t b_s, b_r, b_rho;
  const int rc = goose_spine_budget(B, m, r, rho, &b_s, &b_r, &b_rho);
  if (rc != GOOSE_OK) return rc;

  int n = 0;
  std::vector<int> bdepth(B, 0);
  auto add = [&](int parent, int32_t token, bool spine, int depth) {
    h_tokens[n] = token;
    h_parent[n] = parent;
    h_is_spine[n] = spine ? 1 : 0;
    bdepth[n] = depth;
    return n++;
  };
  auto is_child_token = [&](int parent, int32_t token) {
    for (int i = parent + 1; i < n; ++i)
      if (h_parent[i] == parent && h_tokens[i] == token) return true;
    return false;
  };
  // Attaches up to `count` successors of node p's token (table order, pruned by score, no token
  // twice under one parent); new nodes are appended to `out`.
  auto attach = [&](int p, int count, int depth, std::vector<int>& out) {
    const int32_t t = h_tokens[p];
    if (t < 0 || t >= vocab) return;
    int made = 0;
    for (int k = 0; k < K && made < count && n < B; ++k) {
      const int32_t s = h_succ_ids[(size_t)t * K + k];
      if (s < 0 || !((double)h_succ_scores[(size_t)t * K + k] >= min_score)) continue;
      if (is_child_token(p, s)) continue;
      out.push_back(add(p, s, false, depth));
      ++made;
    }
  };

  add(-1, anchor, true, 0);
  for (int i = 0; i < b_s; ++i) add(i, h_draft[i], true, 0);  // step 1
  std::vector<int> queue;
  attach(0, b_r, 1, queue);                                    // step 2
  if (b_s > 0) {                                               // step 3
    double H = 0.0;
    for (int j = 1; j <= b_s; ++j) H += 1.0 / (double)j;
    for (int i = 1; i <= b_s; ++i) {
      const int a = (int)std::floor((double)b_rho * (1.0 / (double)i) / H);
      attach(i, a, 1, queue);
    }
  }
  for (size_t head = 0; head < queue.size() && n < B; ++head) {  // step 4
    const int v = queue[head];
    if (bdepth[v] >= D) continue;
    attach(v, 1, bdepth[v] + 1, queue);
  }
  *h_n = n;
  return GOOSE_OK;
}

int goose_cycle_mode(int m, int consensus, int bypass_len, int anchor_has_successors) {
  if (m > 0 && (m >= bypass_len || consensus)) return GOOSE_MODE_BYPASS;
  if (m > 0 || anchor_has_successors) return GOOSE_MODE_TREE;
  return GOOSE_MODE_AR;
}

int goose_plan_cycle(const int32_t* h_seq, int n_seq, const int32_t* h_lens, int n_lens, int max_spine, int32_t anchor,
                     const int32_t* h_succ_ids, const float* h_succ_scores, int vocab, int K, int B, double p_hat,
                     double rho, int D, double min_score, int bypass_len, int32_t* h_tokens, int32_t* h_parent,
                     uint8_t* h_is_spine, int32_t* h_n, int32_t* h_mode) {
  if (!h_seq || !h_lens || !h_succ_ids || !h_succ_scores || !h_tokens || !h_parent || !h_is_spine || !h_n || !h_mode)
    return GOOSE_ERR_ARG;
  if (n_seq < 1 || max_spine < 1 || B < 1 + max_spine || B > GOOSE_MAX_B || vocab < 1 || K < 1) return GOOSE_ERR_ARG;
  if (anchor < 0 || anchor >= vocab) return GOOSE_ERR_ARG;
  std::vector<int32_t> draft((size_t)max_spine);
  int32_t m = 0, consensus = 0;
  int rc = goose_context_match(h_seq, n_seq, h_lens, n_lens, max_spine, draft.data(), &m, &consensus);
  if (rc != GOOSE_OK) return rc;
  // does the adjacency table hold a usable successor of the anchor?
  int has_succ = 0;
  for (int k = 0; k < K; ++k) {
    const size_t e = (size_t)anchor * K + k;
    if (h_succ_ids[e] >= 0 && h_succ_scores[e] >= (float)min_score) has_succ = 1;
  }
  const int mode = goose_cycle_mode(m, consensus, bypass_len, has_succ);
  *h_mode = mode;
  if (mode == GOOSE_MODE_BYPASS) {  // the anchor and the whole draft as one chain, every node on the spine
    h_tokens[0] = anchor;
    h_parent[0] = -1;
    h_is_spine[0] = 1;
    for (int i = 0; i < m; ++i) {
      h_tokens[1 + i] = draft[i];
      h_parent[1 + i] = i;
      h_is_spine[1 + i] = 1;
    }
    *h_n = 1 + m;
    return GOOSE_OK;
  }
  if (mode == GOOSE_MODE_TREE)
    return goose_build_spine_tree(anchor, draft.data(), m, h_succ_ids, h_succ_scores, vocab, K, B,
                                  goose_spine_ratio_tier(p_hat), rho, D, min_score, h_tokens, h_parent, h_is_spine, h_n);
  h_tokens[0] = anchor;  // one autoregressive step
  h_parent[0] = -1;
  h_is_spine[0] = 1;
  *h_n = 1;
  return GOOSE_OK;
}

double goose_spine_ratio_tier(double p_hat) { return p_hat < 0.2 ? 0.15 : (p_hat < 0.4 ? 0.30 : 0.50); }

double goose_ema_update(double p_hat, int accepted_spine, int offered_spine, double alpha) {
  if (offered_spine <= 0) return p_hat;
  return (1.0 - alpha) * p_hat + alpha * ((double)accepted_spine / (double)offered_spine);
}

}  // extern "C"
