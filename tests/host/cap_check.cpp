// Prints the resident-workgroup cap and the LDS claim for a plan given as class counts (rows in
// class 32, 31, ..., 0), a slice width in log2 lanes, the active lanes per wave and whether edge weights
// are streamed.  usage: cap_check g_log2 lanes weighted N counts...
#include <cstdio>
#include <cstdlib>

#include "schedule.hpp"

int main(int argc, char** argv) {
  if (argc != 5 + GNNAGG_PLAN_CLASSES) return 2;
  const int g = atoi(argv[1]), lanes = atoi(argv[2]), weighted = atoi(argv[3]);
  const int64_t N = atoll(argv[4]);
  int64_t off[GNNAGG_PLAN_CLASSES + 1];
  off[0] = 0;
  for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k) off[k + 1] = off[k] + atoll(argv[5 + k]);
  const int cap = gnnagg::resident_workgroup_cap(off, N, g, lanes, weighted != 0);
  printf("%d %u %d\n", cap, gnnagg::lds_claim(cap), gnnagg::resident_workgroup_cap(nullptr, N, g, lanes, weighted != 0));
  return 0;
}
