/* Sanitizer driver of the CPU oracle (test infrastructure): rollouts of every game mode under three rule sets (the
 * last one with every rule flag on), both observations.  Built by tests/test_sanitizers.py with
 * -fsanitize=address,undefined; prints one line per configuration and exits 0 when nothing was reported. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "../../oracle/mjo.c"
int main(int argc, char **argv)
{
  const int B = argc > 1 ? atoi(argv[1]) : 64, steps = argc > 2 ? atoi(argv[2]) : 1200;
  unsigned flagsets[3] = {1u | 2u | 4u | 8u, 4u | 8u, 1u | 2u | 4u | 8u | 16u | 32u | 64u | 128u | 256u};
  for (int f = 0; f < 3; f++)
    for (int mode = 0; mode < 3; mode++) {
      MjoRules r;
      memset(&r, 0, sizeof r);
      r.flags = flagsets[f]; r.start_score = 25000; r.illegal_penalty = -1.0f; r.mode = (uint8_t)mode;
      MjoHandle *h;
      if (mjo_create(&h, B, 5, &r)) return 1;
      mjo_step_random(h, steps, 1);
      MjoTokenObs *t = malloc(sizeof(MjoTokenObs) * B * 4);
      unsigned char *obs = malloc((size_t)B * 4 * 56 * 34);
      MjoEnv *ex = malloc(sizeof(MjoEnv) * B);
      mjo_observe_tokens(h, t); mjo_observe(h, obs);
      mjo_export(h, 0, B, ex); mjo_import(h, 0, B, ex);
      mjo_step_random(h, 200, 1);
      printf("oracle flags %u mode %d ok, n_hist[0]=%d\n", r.flags, mode, t[0].n_hist);
      free(t); free(obs); free(ex); mjo_destroy(h);
    }
  return 0;
}
