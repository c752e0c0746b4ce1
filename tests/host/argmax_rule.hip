// Host-side check of the argmax reduction rule the head and commit kernels share (ppsd_device.h: better,
// kNoIndex, argmax_token).  Reads cases from stdin: "vocab n v0 v1 ... v(n-1)" per line ("nan", "inf", "-inf"
// allowed), candidates visited in the order given by a fixed shuffle, prints the token per case.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_2509_19368_amd/csrc/ppsd_device.h"

int main() {
  int vocab, n;
  while (scanf("%d %d", &vocab, &n) == 2) {
    std::vector<float> v(n);
    for (int i = 0; i < n; ++i) {
      char tok[64];
      if (scanf("%63s", tok) != 1) return 2;
      v[i] = !strcmp(tok, "nan") ? NAN : !strcmp(tok, "inf") ? INFINITY : !strcmp(tok, "-inf") ? -INFINITY : (float)atof(tok);
    }
    for (int pass = 0; pass < 2; ++pass) {          // two visiting orders: the result must not depend on it
      float best = -INFINITY;
      int besti = ppsd::kNoIndex;
      for (int k = 0; k < n; ++k) {
        const int i = pass == 0 ? k : (int)(((long long)k * 7919 + 3) % n);
        if (pass == 1 && n % 7919 == 0) break;
        if (ppsd::better(v[i], i, best, besti)) { best = v[i]; besti = i; }
      }
      printf("%d%c", ppsd::argmax_token(besti, vocab), pass == 0 ? ' ' : '\n');
    }
  }
  return 0;
}
