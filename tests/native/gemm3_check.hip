// Checking program for the direct-load GEMM core (gemm_core3.hpp built with DION_GEMM3_BOUNDS): every direct
// load is tested against the address range of an arena that holds all operands; a lane outside it is counted
// and loads nothing.  Results are compared with fp64 sums on the host (small integer inputs: exact in bf16).
//   gemm3_check nt  M r tri_k nseg order  the triangular multiply / Gram form, 256x256 tiles (order = 1: 256x128 tiles,
//                                         costliest column tiles first; 2: that order on 256x256 tiles), up to 3 operand pairs
//   gemm3_check k5  m n r group_n stream  the fused update on 256x128 tiles; stream = 1: the epilogue with the non-temporal hint
//   gemm3_check ks  M N K aks bks nseg lower splitk tail   products whose operands (A if aks, B if bks) are stored with k as
//                                         the slow index and read through the transposing LDS read: the product with
//                                         (M+G)^T (aks = bks = 1), the one with Q (bks = 1), the Gram matrix (both, three
//                                         operand pairs, lower tiles, split over k); tail = 1: a short last round split over k
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

template <bool AKS, bool BKS>
static int run_ks_t(int M, int N, int K, int nseg, int lower, int splitk, int tail) {
  enum { S_A0 = 0, S_A1, S_B0, S_B1, S_OUT, S_PART, S_TAIL, NS = 8 };
  // operand pairs: (A0,B0), (A0,B1), (A1,B0) as in the split-bf16 products (hi hi, hi lo, lo hi)
  const size_t nA = (size_t)M * K, nB = (size_t)N * K, nC = (size_t)M * N;
  std::vector<uint16_t> hA[2], hB[2];
  uint32_t s = 4711;
  auto rnd = [&](int mod) { s = s * 1664525u + 1013904223u; return (int)((s >> 16) % mod) - mod / 2; };
  for (int q = 0; q < (nseg > 1 ? 2 : 1); ++q) {
    hA[q].resize(nA); hB[q].resize(nB);
    for (auto& x : hA[q]) x = f2bf((float)rnd(q ? 3 : 5));
    for (auto& x : hB[q]) x = f2bf((float)rnd(q ? 3 : 5));
  }
  auto al = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off[NS], cur = 0;
  off[S_A0] = cur; cur += al(nA * 2);
  off[S_A1] = cur; cur += nseg > 1 ? al(nA * 2) : 256;
  off[S_B0] = cur; cur += al(nB * 2);
  off[S_B1] = cur; cur += nseg > 1 ? al(nB * 2) : 256;
  const size_t operand_end = cur;
  off[S_OUT] = cur; cur += al(nC * 4);
  off[S_PART] = cur; cur += al(nC * 4 * (splitk > 1 ? splitk : 1));
  off[S_TAIL] = cur; cur += (size_t)256 * 256 * 256 * 4;
  const size_t tab_off = cur; cur += al(NS * sizeof(void*));
  char* arena;
  CK(hipMalloc(&arena, cur));
  CK(hipMemset(arena, 0, cur));
  // device layouts: element (row, k) at [row * K + k] (k fast) or [k * rows + row] (k slow)
  auto upload = [&](int slot, const std::vector<uint16_t>& h, int rows, bool kslow) -> int {
    if (h.empty()) return 0;
    std::vector<uint16_t> t(h.size());
    if (kslow) {   // (blocked, so that neither side of the transposition strides through memory)
      for (int i0 = 0; i0 < rows; i0 += 64)
        for (int k0 = 0; k0 < K; k0 += 64)
          for (int i = i0; i < i0 + 64 && i < rows; ++i)
            for (int k = k0; k < k0 + 64 && k < K; ++k) t[(size_t)k * rows + i] = h[(size_t)i * K + k];
    } else t = h;
    CK(hipMemcpy(arena + off[slot], t.data(), t.size() * 2, hipMemcpyHostToDevice));
    return 0;
  };
  if (upload(S_A0, hA[0], M, AKS) || upload(S_A1, hA[1], M, AKS) || upload(S_B0, hB[0], N, BKS) || upload(S_B1, hB[1], N, BKS)) return 1;
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
  a.splitk = splitk > 1 ? splitk : 1; a.sub_count = 1; a.status_slot = -1; a.noop_slot = -1;
  a.E.colsq_slot = -1; a.side_slot = -1; a.tail_slot = -1; a.E.alpha = 1.f;
  a.M = M; a.N = N; a.K = nseg * K;
  if (nseg > 1) {
    a.nseg = nseg; a.kseg = K;
    a.segA[0] = S_A0; a.segB[0] = S_B0; a.segA[1] = S_A0; a.segB[1] = S_B1; a.segA[2] = S_A1; a.segB[2] = S_B0;
  }
  a.A.slot0 = S_A0; a.A.ld = AKS ? M : K;
  a.B.slot0 = S_B0; a.B.ld = BKS ? N : K;
  a.lower_only = lower;
  a.xcd_remap = 1;
  a.group_n = lower ? 0 : 4;
  if (tail) { a.cus = 256; a.tail_slot = S_TAIL; }
  a.E.slot = splitk > 1 ? S_PART : S_OUT; a.E.ld = N; a.E.split_stride = (long long)nC;
  using Big = TileCfg3<256, 256, 2, 4>;
  if (!gemm3_fits<Big, AKS, BKS>(a)) { printf("does not fit\n"); return 1; }
  printf("launching\n"); fflush(stdout);
  CK((launch_gemm3<Big, false, EPI_STORE, false, AKS, BKS>(a, 1, 0)));
  CK(hipDeviceSynchronize());
  unsigned viol = 0;
  CK(hipMemcpyFromSymbol(&viol, HIP_SYMBOL(dion_gemm3_violations), sizeof(viol)));
  printf("violations %u\n", viol); fflush(stdout);
  const int nparts = splitk > 1 ? splitk : 1;
  std::vector<float> oC(nC * nparts);
  CK(hipMemcpy(oC.data(), arena + off[splitk > 1 ? S_PART : S_OUT], oC.size() * 4, hipMemcpyDeviceToHost));
  long bad = 0, checked = 0;
  auto check = [&](int i, int j) {
    if (lower && j / 256 > i / 256) return;     // tiles above the diagonal are not computed
    double ref = 0;
    for (int sg = 0; sg < nseg; ++sg) {
      const std::vector<uint16_t>& A = hA[sg == 2 ? 1 : 0];
      const std::vector<uint16_t>& B = hB[sg == 1 ? 1 : 0];
      for (int k = 0; k < K; ++k) ref += (double)bf2f(A[(size_t)i * K + k]) * bf2f(B[(size_t)j * K + k]);
    }
    double got = 0;
    for (int q = 0; q < nparts; ++q) got += oC[(size_t)q * nC + (size_t)i * N + j];
    ++checked;
    if (std::fabs(ref - got) > 1e-3 * (1 + std::fabs(ref))) {
      if (bad < 5) printf("mismatch at %d %d: got %g want %g\n", i, j, got, ref);
      ++bad;
    }
  };
  for (int t = 0; t < 20000; ++t) { s = s * 1664525u + 1013904223u; int i = (s >> 8) % M; s = s * 1664525u + 1013904223u; int j = (s >> 8) % N; check(i, j); }
  for (int i = M - 256; i < M; i += 5) for (int j = N - 256; j < N; j += 3) check(i, j);
  printf("checked %ld bad %ld\n", checked, bad);
  return (bad || viol) ? 2 : 0;
}
static int run_ks(int argc, char** argv) {
  const int M = argc > 1 ? atoi(argv[1]) : 4096, N = argc > 2 ? atoi(argv[2]) : 1024, K = argc > 3 ? atoi(argv[3]) : 4096;
  const int aks = argc > 4 ? atoi(argv[4]) : 1, bks = argc > 5 ? atoi(argv[5]) : 1, nseg = argc > 6 ? atoi(argv[6]) : 1;
  const int lower = argc > 7 ? atoi(argv[7]) : 0, splitk = argc > 8 ? atoi(argv[8]) : 1, tail = argc > 9 ? atoi(argv[9]) : 0;
  printf("k-slow operands M=%d N=%d K=%d aks=%d bks=%d nseg=%d lower=%d splitk=%d tail=%d\n", M, N, K, aks, bks, nseg, lower, splitk, tail);
  fflush(stdout);
  if (aks && bks) return run_ks_t<true, true>(M, N, K, nseg, lower, splitk, tail);
  if (!aks && bks) return run_ks_t<false, true>(M, N, K, nseg, lower, splitk, tail);
  printf("unsupported combination\n");
  return 1;
}

int main(int argc, char** argv) {
  if (argc < 2) { printf("usage: gemm3_check nt|k5|ks ...\n"); return 1; }
  if (!strcmp(argv[1], "ks")) return run_ks(argc - 1, argv + 1);
  if (!strcmp(argv[1], "nt")) return run_nt(argc - 1, argv + 1);
  if (!strcmp(argv[1], "k5")) return run_k5(argc - 1, argv + 1);
  printf("unknown mode\n");
  return 1;
}
