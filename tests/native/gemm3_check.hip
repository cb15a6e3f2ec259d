// Checking program for the direct-load GEMM core (gemm_core3.hpp built with DION_GEMM3_BOUNDS): every direct
// load is tested against the address range of an arena that holds all operands; a lane outside it is counted
// and loads nothing.  Results are compared with fp64 sums on the host (small integer inputs: exact in bf16).
//   gemm3_check nt  M r tri_k nseg order  the triangular multiply / Gram form, 256x256 tiles (order = 1: 256x128 tiles,
//                                         costliest column tiles first; 2: that order on 256x256 tiles), up to 3 operand pairs
//   gemm3_check k5  m n r group_n stream  the fused update on 256x128 tiles; stream = 1: the epilogue with the non-temporal hint
// Prints "violations V" and "checked C bad B"; exit status 0 only when V = B = 0.
#define DION_GEMM3_BOUNDS 1
#include "../../paper_2504_05295_amd/csrc/gemm_core3.hpp"
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>
#include <cmath>
using namespace dion;

static uint16_t f2bf(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)(u >> 16); }
static float bf2f(uint16_t h) { uint32_t u = (uint32_t)h << 16; float f; memcpy(&f, &u, 4); return f; }
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
static int run_nt(int argc, char** argv) {
  const int M = argc > 1 ? atoi(argv[1]) : 16384, r = argc > 2 ? atoi(argv[2]) : 1024;
  const int tri = argc > 3 ? atoi(argv[3]) : 1;
  const int nseg = argc > 4 ? atoi(argv[4]) : 3;
  printf("triangular multiply M=%d r=%d tri_k=%d nseg=%d\n", M, r, tri, nseg); fflush(stdout);
  enum { S_P16 = 0, S_ZL16, S_WH16, S_WL16, S_OUT, NS = 8 };
  const size_t nA = (size_t)M * r, nW = (size_t)r * r;
  std::vector<uint16_t> hP(nA), hZ(nA), hWh(nW, 0), hWl(nW, 0);
  uint32_t s = 777;
  auto rnd = [&](int mod) { s = s * 1664525u + 1013904223u; return (int)((s >> 16) % mod) - mod / 2; };
  for (auto& x : hP) x = f2bf((float)rnd(7));
  for (auto& x : hZ) x = f2bf((float)rnd(3));
  for (int j = 0; j < r; ++j)
    for (int k = 0; k <= (tri ? j : r - 1); ++k) { hWh[(size_t)j * r + k] = f2bf((float)rnd(5)); hWl[(size_t)j * r + k] = f2bf((float)rnd(3)); }
  // arena: [P16][ZL16][WH16][WL16][OUT fp32][table]
  auto al = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off[8], cur = 0;
  off[S_P16] = cur; cur += al(nA * 2);
  off[S_ZL16] = cur; cur += al(nA * 2);
  off[S_WH16] = cur; cur += al(nW * 2);
  off[S_WL16] = cur; cur += al(nW * 2);
  const size_t operand_end = cur;
  off[S_OUT] = cur; cur += al(nA * 4);
  const size_t tab_off = cur; cur += al(NS * sizeof(void*));
  char* arena;
  CK(hipMalloc(&arena, cur));
  CK(hipMemset(arena, 0, cur));
  CK(hipMemcpy(arena + off[S_P16], hP.data(), nA * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_ZL16], hZ.data(), nA * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_WH16], hWh.data(), nW * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_WL16], hWl.data(), nW * 2, hipMemcpyHostToDevice));
  void* htab[NS] = {};
  for (int i = 0; i <= S_OUT; ++i) htab[i] = arena + off[i];
  CK(hipMemcpy(arena + tab_off, htab, sizeof(htab), hipMemcpyHostToDevice));
  unsigned long long bounds[2] = {(unsigned long long)arena, (unsigned long long)arena + operand_end};
  unsigned zero = 0;
  CK(hipMemcpyToSymbol(HIP_SYMBOL(dion_gemm3_bounds), bounds, sizeof(bounds)));
  CK(hipMemcpyToSymbol(HIP_SYMBOL(dion_gemm3_violations), &zero, sizeof(zero)));

  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.table = (void* const*)(arena + tab_off);
  a.nslots = NS;
  a.splitk = 1; a.sub_count = 1; a.status_slot = -1;
  a.noop_slot = -1;
  a.E.colsq_slot = -1;
  a.side_slot = -1;
  a.E.alpha = 1.f;
  a.M = M; a.N = r; a.K = nseg * r;
  a.nseg = nseg; a.kseg = r;
  a.segA[0] = S_P16; a.segB[0] = S_WH16;
  a.segA[1] = S_P16; a.segB[1] = S_WL16;
  a.segA[2] = S_ZL16; a.segB[2] = S_WH16;
  a.A.slot0 = S_P16; a.A.ld = r;
  a.B.slot0 = S_WH16; a.B.ld = r;
  a.tri_k = tri;
  a.E.slot = S_OUT; a.E.ld = r;
  a.xcd_remap = 1;
  const int order = argc > 5 ? atoi(argv[5]) : 0;   // 1: 256x128 tiles, costliest column tiles first; 2: that order on 256x256 tiles
  const int narrow = order == 1;
  using Cfg = TileCfg3<256, 256, 2, 4>;
  using Narrow = TileCfg3<256, 128, 4, 2>;
  a.heavy_first = order != 0;
  if (narrow ? !gemm3_fits<Narrow>(a) : !gemm3_fits<Cfg>(a)) { printf("does not fit\n"); return 1; }
  printf("launching\n"); fflush(stdout);
  if (narrow) CK((launch_gemm3<Narrow, false, EPI_STORE, false>(a, 1, 0)));
  else CK((launch_gemm3<Cfg, false, EPI_STORE, false>(a, 1, 0)));
  CK(hipDeviceSynchronize());
  unsigned viol = 0;
  CK(hipMemcpyFromSymbol(&viol, HIP_SYMBOL(dion_gemm3_violations), sizeof(viol)));
  unsigned long long first[64];
  CK(hipMemcpyFromSymbol(first, HIP_SYMBOL(dion_gemm3_first), sizeof(first)));
  printf("violations %u\n", viol);
  if (viol) {
    printf("arena %p\n", (void*)arena);
    for (int v = 0; v < 16 && v < (int)viol; ++v)
      printf("viol %d: base %#llx voff %llu lds %#llx block %llu thread %llu\n", v, first[4 * v], first[4 * v + 1], first[4 * v + 2], first[4 * v + 3] / 1024, first[4 * v + 3] % 1024);
    for (int i = 0; i <= S_OUT; ++i) printf("  slot %d at arena + %zu\n", i, off[i]);
  }
  fflush(stdout);
  std::vector<float> hC(nA);
  CK(hipMemcpy(hC.data(), arena + off[S_OUT], nA * 4, hipMemcpyDeviceToHost));
  long bad = 0, checked = 0;
  auto check = [&](int i, int j) {
    double ref = 0;
    for (int k = 0; k < r; ++k) {
      const double p = bf2f(hP[(size_t)i * r + k]), z = bf2f(hZ[(size_t)i * r + k]);
      const double wh = bf2f(hWh[(size_t)j * r + k]), wl = bf2f(hWl[(size_t)j * r + k]);
      ref += p * wh + (nseg > 1 ? p * wl : 0) + (nseg > 2 ? z * wh : 0);
    }
    ++checked;
    if (std::fabs(ref - hC[(size_t)i * r + j]) > 1e-3 * (1 + std::fabs(ref))) {
      if (bad < 5) printf("mismatch at %d %d: got %g want %g\n", i, j, hC[(size_t)i * r + j], ref);
      ++bad;
    }
  };
  for (int t = 0; t < 20000; ++t) { s = s * 1664525u + 1013904223u; int i = (s >> 8) % M; s = s * 1664525u + 1013904223u; int j = (s >> 8) % r; check(i, j); }
  for (int i = M - 256; i < M; ++i) for (int j = 0; j < r; j += 7) check(i, j);
  printf("checked %ld bad %ld\n", checked, bad);
  return (bad || viol) ? 2 : 0;
}

static int run_k5(int argc, char** argv) {
  const int m = argc > 1 ? atoi(argv[1]) : 2048, n = argc > 2 ? atoi(argv[2]) : 4096, r = argc > 3 ? atoi(argv[3]) : 2048;
  const int group_n = argc > 4 ? atoi(argv[4]) : 0;
  printf("fused update m=%d n=%d r=%d group_n=%d\n", m, n, r, group_n); fflush(stdout);
  enum { S_P16 = 0, S_R16, S_Q16, S_X, S_G, S_M, S_STATUS, NS = 8 };
  const size_t nP = (size_t)m * r, nR = (size_t)n * r, nX = (size_t)m * n;
  std::vector<uint16_t> hP(nP), hR(nR), hQ(nR), hG(nX);
  std::vector<float> hX(nX), hM(nX);
  uint32_t s = 4242;
  auto rnd = [&](int mod) { s = s * 1664525u + 1013904223u; return (int)((s >> 16) % mod) - mod / 2; };
  for (auto& x : hP) x = f2bf((float)rnd(5));
  for (auto& x : hR) x = f2bf((float)rnd(7));
  for (auto& x : hQ) x = f2bf((float)rnd(3));
  for (auto& x : hG) x = f2bf((float)rnd(9));
  for (auto& x : hX) x = (float)rnd(11);
  for (auto& x : hM) x = (float)rnd(13);
  auto al = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off[NS], cur = 0;
  off[S_P16] = cur; cur += al(nP * 2);
  off[S_R16] = cur; cur += al(nR * 2);
  off[S_Q16] = cur; cur += al(nR * 2);
  const size_t operand_end = cur;
  off[S_X] = cur; cur += al(nX * 4);
  off[S_G] = cur; cur += al(nX * 2);
  off[S_M] = cur; cur += al(nX * 4);
  off[S_STATUS] = cur; cur += 256;
  const size_t tab_off = cur; cur += al(NS * sizeof(void*));
  char* arena;
  CK(hipMalloc(&arena, cur));
  CK(hipMemset(arena, 0, cur));
  CK(hipMemcpy(arena + off[S_P16], hP.data(), nP * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_R16], hR.data(), nR * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_Q16], hQ.data(), nR * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_X], hX.data(), nX * 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_G], hG.data(), nX * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(arena + off[S_M], hM.data(), nX * 4, hipMemcpyHostToDevice));
  void* htab[NS] = {};
  for (int i = 0; i < NS - 1; ++i) htab[i] = arena + off[i];
  CK(hipMemcpy(arena + tab_off, htab, sizeof(htab), hipMemcpyHostToDevice));
  unsigned long long bounds[2] = {(unsigned long long)arena, (unsigned long long)arena + operand_end};
  unsigned zero = 0;
  CK(hipMemcpyToSymbol(HIP_SYMBOL(dion_gemm3_bounds), bounds, sizeof(bounds)));
  CK(hipMemcpyToSymbol(HIP_SYMBOL(dion_gemm3_violations), &zero, sizeof(zero)));
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.table = (void* const*)(arena + tab_off);
  a.nslots = NS;
  a.splitk = 1; a.sub_count = 1; a.status_slot = S_STATUS;
  a.noop_slot = -1;
  a.E.colsq_slot = -1;
  a.side_slot = -1;
  a.E.alpha = 1.f;
  a.M = m; a.N = n; a.K = r;
  a.A.slot0 = S_P16; a.A.ld = r;
  a.B.slot0 = S_R16; a.B.ld = r;
  a.B2.slot0 = S_Q16; a.B2.ld = r;
  a.E.slotX = S_X; a.E.slotG = S_G; a.E.slotM = S_M; a.E.ld = n;
  a.E.c_m = 0.5f; a.E.c_x = 0.25f;
  a.xcd_remap = 1;
  a.group_n = group_n;
  const int stream = argc > 5 ? atoi(argv[5]) : 0;
  using Big = TileCfg3<256, 128, 2, 4>;
  if (!gemm3_fits<Big>(a)) { printf("does not fit\n"); return 1; }
  printf("launching\n"); fflush(stdout);
  if (stream) CK((launch_gemm3<Big, true, EPI_UPDATE_STREAM, true>(a, 1, 0)));
  else CK((launch_gemm3<Big, true, EPI_UPDATE, true>(a, 1, 0)));
  CK(hipDeviceSynchronize());
  unsigned viol = 0;
  CK(hipMemcpyFromSymbol(&viol, HIP_SYMBOL(dion_gemm3_violations), sizeof(viol)));
  printf("violations %u\n", viol); fflush(stdout);
  std::vector<float> oX(nX), oM(nX);
  CK(hipMemcpy(oX.data(), arena + off[S_X], nX * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(oM.data(), arena + off[S_M], nX * 4, hipMemcpyDeviceToHost));
  long bad = 0, checked = 0;
  auto check = [&](int i, int j) {
    double pr = 0, pq = 0;
    for (int k = 0; k < r; ++k) {
      const double p = bf2f(hP[(size_t)i * r + k]);
      pr += p * bf2f(hR[(size_t)j * r + k]);
      pq += p * bf2f(hQ[(size_t)j * r + k]);
    }
    const size_t e = (size_t)i * n + j;
    const double mref = (double)hM[e] + bf2f(hG[e]) - 0.5 * pr, xref = (double)hX[e] - 0.25 * pq;
    ++checked;
    if (std::fabs(mref - oM[e]) > 1e-3 * (1 + std::fabs(mref)) || std::fabs(xref - oX[e]) > 1e-3 * (1 + std::fabs(xref))) {
      if (bad < 5) printf("mismatch at %d %d: M got %g want %g, X got %g want %g\n", i, j, oM[e], mref, oX[e], xref);
      ++bad;
    }
  };
  for (int t = 0; t < 20000; ++t) { s = s * 1664525u + 1013904223u; int i = (s >> 8) % m; s = s * 1664525u + 1013904223u; int j = (s >> 8) % n; check(i, j); }
  for (int i = m - 256; i < m; i += 3) for (int j = n - 128; j < n; ++j) check(i, j);
  printf("checked %ld bad %ld\n", checked, bad);
  return (bad || viol) ? 2 : 0;
}

int main(int argc, char** argv) {
  if (argc < 2) { printf("usage: gemm3_check nt|k5 ...\n"); return 1; }
  if (!strcmp(argv[1], "nt")) return run_nt(argc - 1, argv + 1);
  if (!strcmp(argv[1], "k5")) return run_k5(argc - 1, argv + 1);
  printf("unknown mode\n");
  return 1;
}
