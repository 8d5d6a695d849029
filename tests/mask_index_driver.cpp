// Host-only driver around csrc/mask_index.h for the sanitizer test: built with
// -fsanitize=address,undefined by tests/test_mask_index_sanitized.py, it prints what the
// library's integer index code returns so that the test can compare it with masks
// built from the paper's prose (sections 4.1, 4.2) by the oracle.  No GPU, no HIP.
//
// stdin, one case per line:
//   G S L k eps tq tk t     whole grids: row limits, first seeing query, tile classes, bands
//   P p j k eps L t         single positions (sizes near the top of the int32 range)
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include "../paper_2505_24544_amd/csrc/mask_index.h"

using namespace beagle;

int main() {
  char kind;
  while (scanf(" %c", &kind) == 1) {
    if (kind == 'G') {
      int S, L, k, eps, tq, tk, t;
      if (scanf("%d %d %d %d %d %d %d", &S, &L, &k, &eps, &tq, &tk, &t) != 7) return 2;
      MaskParams mp{k, eps, L, 0};
      std::vector<int32_t> lim((size_t)S), fq((size_t)L);      // heap: out-of-range indices trip the sanitizer
      for (int p = 0; p < S; ++p) lim[(size_t)p] = row_limit(p, mp);
      for (int j = 0; j < L; ++j) fq[(size_t)j] = first_query_seeing(j, mp);
      printf("G %d %d %d %d %d %d %d\n", S, L, k, eps, tq, tk, t);
      printf("lim");
      for (int p = 0; p < S; ++p) printf(" %d", lim[(size_t)p]);
      printf("\nfq");
      for (int j = 0; j < L; ++j) printf(" %d", fq[(size_t)j]);
      printf("\ncls");
      for (int q0 = 0; q0 < S; q0 += tq)
        for (int j0 = 0; j0 < L; j0 += tk)
          printf(" %d", (int)tile_class(q0, q0 + tq < S ? q0 + tq : S, j0, j0 + tk < L ? j0 + tk : L, mp));
      printf("\nband");
      for (int p = 0; p < S; ++p) {
        int32_t lo, hi;
        sim_band(p, k, eps, t, L, lo, hi);
        printf(" %d %d", lo, hi);
      }
      printf("\n");
    } else if (kind == 'P') {
      int p, j, k, eps, L, t;
      if (scanf("%d %d %d %d %d %d", &p, &j, &k, &eps, &L, &t) != 6) return 2;
      MaskParams mp{k, eps, L, 0};
      int32_t lo, hi;
      sim_band(p, k, eps, t, L, lo, hi);
      printf("P %d %d %d %d %d %d\n", row_limit(p, mp), first_query_seeing(j, mp), window_start(p, k, eps),
             window_start_raw(p, k, eps), lo, hi);
    } else {
      return 2;
    }
  }
  return 0;
}
