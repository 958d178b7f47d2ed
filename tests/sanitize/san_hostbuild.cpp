// Sanitizer driver of the TEST-ONLY host build of the kernels' per-environment code: rollouts of every game mode
// under three rule sets (the last one with every rule flag on), both observations, export and import.  Built by
// tests/test_sanitizers.py with AddressSanitizer + UndefinedBehaviorSanitizer and, where clang offers it, with
// MemorySanitizer (uninitialised reads), once with every function inlined as in the kernels and once with every
// function out of line (-DSAN_OUT_OF_LINE).
#ifdef SAN_OUT_OF_LINE
#define MJ_HD inline __attribute__((noinline))
#endif
#include "../hostsim/hostsim.cpp"
#include <cstdio>
int main(int argc, char **argv)
{
  const int B = argc > 1 ? atoi(argv[1]) : 64, steps = argc > 2 ? atoi(argv[2]) : 1200;
  unsigned flagsets[3] = {1u | 2u | 4u | 8u, 4u | 8u, 511u};
  for (int f = 0; f < 3; f++)
    for (int mode = 0; mode < 3; mode++) {
      MjRules r;
      memset(&r, 0, sizeof r);
      r.flags = flagsets[f]; r.start_score = 25000; r.illegal_penalty = -1.0f; r.mode = (uint8_t)mode;
      Sim *h = hs_create(B, 5, &r);
      hs_step_random(h, steps, 1);
      std::vector<MjTokenObs> t((size_t)B * 4);
      std::vector<uint8_t> obs((size_t)B * 4 * 56 * 34);
      std::vector<MjEnvCanon> ex(B);
      hs_observe_tokens(h, t.data()); hs_observe(h, obs.data()); hs_export(h, 0, B, ex.data());
      hs_import(h, 0, B, ex.data());
      hs_step_random(h, 200, 1);
      printf("host build flags %u mode %d ok, n_hist[0]=%d\n", r.flags, mode, t[0].n_hist);
      hs_destroy(h);
    }
  return 0;
}
