// Replays a script of cache operations on the library's host-side n-gram table (plain C++, built with
// AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_host_table_sanitized.py) and prints the table's state
// at every "dump", for comparison with the CPU oracle.  Script, one operation per line:
//   init <capacity> <policy> <max_len>
//   insert <n> then n lines "<len> <ids...> <target>"
//   import <n> then n lines "<len> <ids...> <target> <uses> <last_used>"
//   step <n> then n lines "<len> <ids...>"            one verification step that used these keys (with multiplicity)
//   offsets <B> <max_k> <B+1 values>                  runs the row-offset check, prints its result
//   dump
#include <cstdio>
#include <cstdlib>
#include <iostream>
#include <string>
#include <vector>

#include "ngram_table.h"

using namespace otv;

struct Csr {
  std::vector<int32_t> off{0}, ids, targets;
  std::vector<int64_t> uses, last;
};

static Csr read_items(int n, bool with_target, bool with_stats) {
  Csr c;
  for (int e = 0; e < n; ++e) {
    int len;
    std::cin >> len;
    for (int i = 0; i < len; ++i) { int v; std::cin >> v; c.ids.push_back(v); }
    c.off.push_back((int32_t)c.ids.size());
    if (with_target) { int t; std::cin >> t; c.targets.push_back(t); }
    if (with_stats) { long long u, l; std::cin >> u >> l; c.uses.push_back(u); c.last.push_back(l); }
  }
  return c;
}

int main() {
  NgramTable tab;
  std::string op;
  int V_d = 1 << 30, V_t = 1 << 30;
  while (std::cin >> op) {
    if (op == "init") {
      int cap, policy, max_len;
      std::cin >> cap >> policy >> max_len;
      tab.init(cap, policy, max_len);
    } else if (op == "insert") {
      int n; std::cin >> n;
      Csr c = read_items(n, true, false);
      const char* what = "";
      if (check_entries(n, c.off.data(), c.ids.data(), c.targets.data(), tab.max_len(), V_d, V_t, &what)) { printf("rejected %s\n", what); continue; }
      const int64_t fresh = tab.count_fresh(n, c.off.data(), c.ids.data());
      if (tab.size() + fresh > tab.capacity() && (tab.policy() == kPolicyNone || tab.capacity() == 0)) { printf("full\n"); continue; }
      const int ev = tab.insert(n, c.off.data(), c.ids.data(), c.targets.data());
      printf("evicted %d dirty %zu\n", ev, tab.take_dirty().size());
    } else if (op == "import") {
      int n; std::cin >> n;
      Csr c = read_items(n, true, true);
      const int64_t fresh = tab.count_fresh(n, c.off.data(), c.ids.data());
      if (tab.size() + fresh > tab.capacity()) { printf("full\n"); continue; }
      tab.import_entries(n, c.off.data(), c.ids.data(), c.targets.data(), c.uses.data(), c.last.data());
      printf("imported %d dirty %zu\n", n, tab.take_dirty().size());
    } else if (op == "step") {
      int n; std::cin >> n;
      Csr c = read_items(n, false, false);
      tab.tick();
      for (int e = 0; e < n; ++e) {
        const int64_t s = tab.lookup(c.ids.data() + c.off[e], c.off[e + 1] - c.off[e]);
        if (s < 0 || !tab.record_use((uint32_t)s, tab.clock())) { printf("unknown key in step\n"); return 2; }
      }
    } else if (op == "offsets") {
      int B, max_k; std::cin >> B >> max_k;
      std::vector<int32_t> off(B + 1);
      for (auto& v : off) std::cin >> v;
      const char* what = "";
      printf("offsets %d\n", check_row_offsets(B, off.data(), max_k, &what));
    } else if (op == "dump") {
      const std::string bad = tab.check();
      if (!bad.empty()) { printf("INVARIANT %s\n", bad.c_str()); return 3; }
      const int n = tab.size();
      std::vector<int32_t> off(n + 1), ids((size_t)tab.total_key_ids() + 1), targets(n + 1);
      std::vector<int64_t> uses(n + 1), last(n + 1);
      tab.export_entries(off.data(), ids.data(), targets.data(), uses.data(), last.data());
      printf("state clock %u n %d\n", tab.clock(), n);
      for (int e = 0; e < n; ++e) {
        printf("entry");
        for (int i = off[e]; i < off[e + 1]; ++i) printf(" %d", ids[i]);
        printf(" -> %d uses %lld last %lld\n", targets[e], (long long)uses[e], (long long)last[e]);
      }
      printf("end\n");
    } else {
      fprintf(stderr, "unknown operation %s\n", op.c_str());
      return 1;
    }
  }
  return 0;
}
