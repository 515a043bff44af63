// Host-side check of the fused backward GEMM's row loads (launch.hpp: fused_seg0_step, fused_row, fused_code_offset,
// fused_const_offset): for many shapes, every load the kernel's schedule asks for lies inside the packed codes
// (N x K0 / 2 bytes) and the constants (N x K0 / 64 floats), and the step counter that the unrolled steady-state loop
// advances by one per iteration equals the clamped formula the other iterations evaluate.
// The schedule replayed here is the kernel's: the prologue loads tiles KT1, 1, 2, 3; iteration k (k = 0 .. KT - 2)
// loads tile k + 4; iterations run five at a time without clamping while k + 8 < KT.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "launch.hpp"

using namespace qlora;

static long long checked = 0;

static bool load_ok(int N, int KT0, int n0, int tid, int step) {
  if (step < 0 || step >= KT0) return false;
  const int row = fused_row(n0, tid, N);
  if (row < 0 || row >= N) return false;
  const int64_t q = fused_code_offset(row, step, KT0), c = fused_const_offset(row, step, KT0);
  ++checked;
  return q >= 0 && q + 32 <= (int64_t)N * KT0 * 32 && c >= 0 && c + 4 <= (int64_t)N * KT0 * 4 && q < (1ll << 31);
}

static bool check_shape(int N, int K0, int K1) {
  if (!gemm_nt_fused_fits(K0, K1, N)) return true;            // the launcher refuses it
  const int KT0 = K0 / 64, KT1 = K1 / 64, KT = KT0 + KT1;
  const int tiles_n = (N + 255) / 256;
  for (int tn : {0, tiles_n / 2, tiles_n - 1}) {
    const int n0 = tn * 256;
    for (int tid : {0, 1, 63, 64, 127, 255}) {
      // prologue
      for (int t : {KT1, 1, 2, 3})
        if (!load_ok(N, KT0, n0, tid, fused_seg0_step(t, KT, KT1))) return false;
      int kq = 4 - KT1, k = 0;
      while (k + 8 < KT) {                                    // steady state: five iterations, counter advanced by one
        for (int i = 0; i < 5; ++i) {
          if (kq != fused_seg0_step(k + 4, KT, KT1)) return false;
          if (!load_ok(N, KT0, n0, tid, kq)) return false;
          ++kq; ++k;
        }
      }
      for (; k + 1 < KT; ++k)                                 // the other iterations evaluate the clamped formula
        if (!load_ok(N, KT0, n0, tid, fused_seg0_step(k + 4, KT, KT1))) return false;
    }
  }
  return true;
}

int main() {
  int shapes = 0;
  for (int N : {4, 64, 192, 256, 260, 448, 1024, 8192, 22016})
    for (int KT0 = 1; KT0 <= 400; KT0 += (KT0 < 24 ? 1 : 47))
      for (int K1 : {0, 64}) {
        if (!check_shape(N, KT0 * 64, K1)) { std::printf("FAIL N=%d K0=%d K1=%d\n", N, KT0 * 64, K1); return 1; }
        ++shapes;
      }
  // what the launcher must refuse
  if (gemm_nt_fused_fits(8192, 128, 1024) || gemm_nt_fused_fits(100, 0, 1024) || gemm_nt_fused_fits(0, 0, 8) ||
      gemm_nt_fused_fits(1 << 20, 0, 1 << 14)) { std::printf("FAIL fits\n"); return 1; }
  std::printf("OK %d shapes %lld loads\n", shapes, checked);
  return 0;
}
