// Host-side check of the work partition of the few-token list kernels (no GPU needed): for many shape lists the
// plan's ranges must tile the line of units exactly, be ascending with empty ranges only at the two ends, list_rho_of
// must invert list_start, and the number of workgroups that share a slab (brute force over the ranges) must equal what the
// kernels derive from the formula, stay within an arrival word's 23 bits and within the plan's buffer sizes.
// Prints "OK <plans>" or the first violation.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "launch.hpp"

using namespace qlora;

static int fail(const char* what, int a, int b, int c) {
  std::printf("FAIL %s (%d, %d, %d)\n", what, a, b, c);
  return 1;
}

static int check(bool bwd, int M, int n, const int* h, const int* o, const int* r) {
  const ListPlan P = fewlist_plan(bwd, M, n, h, o, r);
  if (!P.ok) return -1;
  const ListPart& q = P.part;
  if (q.grid < 1 || q.grid > 256) return fail("grid", q.grid, 0, 0);
  if (list_start(q, 0) != 0 || list_start(q, q.grid) != P.total_units) return fail("ends", list_start(q, q.grid), P.total_units, 0);
  // ascending; empty ranges only before the first and after the last non-empty one (a workgroup between two
  // contributors of a slab that contributes nothing would be waited for in that slab's arrival word)
  int first_full = -1, last_full = -1;
  for (int rho = 0; rho < q.grid; ++rho) {
    const int a = list_start(q, rho), b = list_start(q, rho + 1);
    if (b < a) return fail("descending range", rho, a, b);
    if (b > a) { if (first_full < 0) first_full = rho; last_full = rho; }
  }
  if (first_full < 0) return fail("no work at all", 0, 0, 0);
  for (int rho = first_full; rho <= last_full; ++rho)
    if (list_start(q, rho + 1) <= list_start(q, rho)) return fail("empty range between contributors", rho, first_full, last_full);
  for (int rho = first_full; rho <= last_full; ++rho) {
    const int a = list_start(q, rho), b = list_start(q, rho + 1);
    if (list_rho_of(q, a) != rho || list_rho_of(q, b - 1) != rho) return fail("rho_of", rho, a, b);
  }
  for (int u = 0; u < P.total_units; u += 1 + P.total_units / 997) {   // inverse map on a sample of all units
    const int rho = list_rho_of(q, u);
    if (rho < 0 || rho >= q.grid || list_start(q, rho) > u || list_start(q, rho + 1) <= u) return fail("rho_of(u)", u, rho, 0);
  }
  int slabs = 0, adapters = 0;
  for (int l = 0; l < n; ++l) {
    const int outs = bwd ? h[l] : o[l], contr = bwd ? o[l] : h[l];
    if (P.n_slabs[l] != (outs + 255) / 256) return fail("n_slabs", l, P.n_slabs[l], outs);
    if (P.ups[l] != (bwd ? (contr + 127) / 128 : (contr + 15) / 16)) return fail("ups", l, P.ups[l], contr);
    if (P.ctr0[l] != slabs || P.a0[l] != adapters) return fail("offsets", l, P.ctr0[l], P.a0[l]);
    if (r[l] > 0) {
      if (P.n_lparts[l] < 1 || P.n_lparts[l] > 23) return fail("n_lparts", l, P.n_lparts[l], 0);
      if ((long long)P.n_lparts[l] * P.lora_chunk[l] < contr || (long long)(P.n_lparts[l] - 1) * P.lora_chunk[l] >= contr)
        return fail("adapter chunks do not tile the contraction", l, P.n_lparts[l], P.lora_chunk[l]);
    } else if (P.n_lparts[l] != 0) return fail("adapter items without an adapter", l, 0, 0);
    for (int s = 0; s < P.n_slabs[l]; ++s) {
      const int U0 = P.unit0[l] + s * P.ups[l], U1 = U0 + P.ups[l];
      int brute = 0;
      for (int rho = 0; rho < q.grid; ++rho)
        if (list_start(q, rho) < U1 && list_start(q, rho + 1) > U0) ++brute;
      const int formula = list_rho_of(q, U1 - 1) - list_rho_of(q, U0) + 1;
      if (brute != formula) return fail("contributors", l, brute, formula);
      if (formula > 23 || formula > P.max_contrib[l]) return fail("too many contributors", l, formula, P.max_contrib[l]);
    }
    if (P.part_floats[l] != (size_t)P.n_slabs[l] * P.max_contrib[l] * M * 256) return fail("part size", l, 0, 0);
    slabs += P.n_slabs[l];
    adapters += P.n_lparts[l];
  }
  if (q.n_adapter != adapters || slabs != P.total_slabs || slabs > 2046) return fail("totals", adapters, slabs, 0);
  return 0;
}

int main() {
  int plans = 0;
  unsigned long long state = 0x9E3779B97F4A7C15ull;
  auto rnd = [&](int m) { state = state * 6364136223846793005ull + 1442695040888963407ull; return (int)((state >> 33) % (unsigned)m); };
  // the shapes the benchmark and the tests run
  {
    const int h[7] = {8192, 8192, 8192, 8192, 8192, 8192, 22016}, o[7] = {8192, 8192, 8192, 8192, 22016, 22016, 8192};
    const int r[7] = {64, 64, 64, 64, 64, 64, 64};
    for (int bwd = 0; bwd < 2; ++bwd)
      for (int M : {1, 4, 16}) {
        const int rc = check(bwd, M, 7, h, o, r);
        if (rc) return rc < 0 ? fail("the 65B block is not plannable", bwd, M, 0) : rc;
        ++plans;
      }
  }
  for (int it = 0; it < 4000; ++it) {
    int h[kListMax], o[kListMax], r[kListMax];
    const int n = 1 + rnd(kListMax), M = 1 + rnd(16);
    for (int l = 0; l < n; ++l) {
      const int big = rnd(4);
      h[l] = 64 * (1 + rnd(big == 0 ? 400 : big == 1 ? 40 : 4));
      o[l] = 64 * (1 + rnd(big == 0 ? 4 : big == 1 ? 40 : 400));
      r[l] = 16 * rnd(5);
    }
    const int rc = check(rnd(2), M, n, h, o, r);
    if (rc > 0) return rc;
    if (rc == 0) ++plans;
  }
  std::printf("OK %d\n", plans);
  return 0;
}
