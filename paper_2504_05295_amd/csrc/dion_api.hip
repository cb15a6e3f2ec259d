// C ABI of libdion.so and the host-side sequencing of one Dion step (see include/dion.h).
//
// Sequence per shape group (Algorithm 1 + unsharded update rule + PowerIter1 of the paper; the
// data-parallel all-reduces of PowerIter1 are absent because everything runs on one GPU):
//   K1  Z = (M+G) Q                      MFMA GEMM; M+G fused into the operand load, or (shapes that fill the GPU with
//                                        256-wide tiles) read from the one bf16 copy of M+G that a pass writes first
//   orth: CholeskyQR2 (Appendix A applied twice): Gram, blocked Cholesky, triangular inverse, Z L^-T
//   K2  R = (M+G)^T P                    MFMA GEMM; the operand is transposed on its way into the registers (from
//                                        M and G, or from the same bf16 copy through transposing LDS reads)
//   K6  s_j = ||R_j||, d_j = 1/(s_j + eps);   K7  Q = R diag(d)
//   K5  M = (M+G) - (1-mu) P R^T ;  X = X - eta sqrt(m/n) P Q^T     one fused pass
// The stages are functions of their own (stage_k1, stage_orth, ...); the Dion step, its transposed form, the
// Lazy-Dion step and the two stages of Double Dion are different sequences of them.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/dion.h"
#include "internal.hpp"

using namespace dion;

namespace dion {
int pick_variant(long long M, long long N, long long K, long long batch, bool aligned) {
  const bool big_ok = aligned && M % 128 == 0 && N % 128 == 0 && K % 32 == 0;
  const bool small_ok = aligned && M % 64 == 0 && N % 64 == 0 && K % 64 == 0;
  if (big_ok) {
    const long long tiles = (M / 128) * (N / 128) * batch;
    return (tiles >= 256 || !small_ok) ? VAR_BIG : VAR_SMALL;
  }
  return small_ok ? VAR_SMALL : VAR_SMALL_CHECKED;
}
void plan_chol_grid(int cus, int batch, int nb, int* pr, int* pc, int* chain) {
  *pr = 0; *pc = 0; *chain = 0;
  if (cus < 1 || batch < 1 || nb < 4 || nb > 128) return;
  // From two workgroups per matrix on the single launch still beats a launch per panel, in which every workgroup redoes
  // the diagonal block and the second pass costs a launch per panel to skip.  With sixteen and more per matrix one of
  // them carries the whole chain of diagonal blocks and the others (pr x pc, coprime) help.
  const int per = cus / batch;
  if (per >= 256 && nb >= 16) { *pr = 15; *pc = 17; *chain = 1; }
  else if (per >= 64) { *pr = 7; *pc = 9; *chain = 1; }
  else if (per >= 16) { *pr = 3; *pc = 5; *chain = 1; }
  else if (per >= 8) { *pr = 4; *pc = 2; }
  else if (per >= 4) { *pr = 2; *pc = 2; }
  else if (per >= 2) { *pr = 2; *pc = 1; }
  const long long groups = (long long)*pr * *pc + *chain;
  if (groups * batch > cus || groups > INV_TREE_MAX_GROUPS) { *pr = 0; *pc = 0; *chain = 0; }
}
}  // namespace dion

namespace {

struct Entry {
  int64_t m, n, r;
  int form;   // DION_FORM_*
  int group;
  int row;  // row of the pointer table (group-sorted order)
};
// byte offsets of the workspace slots of one matrix
struct Carve {
  size_t off[NSLOTS];
  size_t total;
};
// How the Gram matrix of a rows x r matrix is split over the contraction (fixed at init: sizes workspace).
struct GramPlan {
  int variant, splitk, kps;   // fp32 path: tile variant, number of splits, rows per split
  int splitk2;                // split-bf16 path on large tiles
  int split_cap256;           // most partial results the 256 x 256-tile kernel may be asked for (sizes their buffer)
};
struct Group {
  int64_t m, n, r;
  int form;        // DION_FORM_*: all matrices of a group share it
  int rp;          // r rounded up to a multiple of CHOL_NB
  int first_row, count;
  GramPlan gram_m, gram_n;   // Gram products over the m x r matrices of a Dion step / the n x r ones of a Lazy-Dion refresh
  int k12_splitk;     // split-K of K1 / K2 on the large-tile path when their outputs have too few tiles
  bool direct12;      // K1 / K2 may read bf16(M + G) from memory (direct-load kernels): the shape fills the GPU with
                      // 256 x 256 tiles and the copy fits the kernels' 32-bit offsets
  bool big;           // the large-tile bf16 kernels serve this group (bf16 operand mode, tile-aligned shape): only then
                      // are the bf16 operand copies carved
  size_t bytes_per_entry;
  Carve carve;     // slot offsets inside one matrix' share of the workspace
  size_t ws_off;   // offset of the group's first matrix in the workspace (set by dion_init_state)
};

constexpr int kEventsPerGroup = 2 * DION_STAGE_COUNT;
constexpr int K1_PARTS = 4;   // parts of the contraction of K1 when the bf16 copy of M + G is made alongside it   // a start and an end event per stage

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int padded_rank(int64_t r) { return (int)((r + CHOL_NB - 1) / CHOL_NB * CHOL_NB); }

GramPlan plan_gram_rows(const Group& g, int64_t rows) {
  GramPlan gp;
  gp.variant = pick_variant(g.r, g.r, rows, g.count, true);
  const int bt = (gp.variant == VAR_BIG) ? 128 : 64;
  const int bk = (gp.variant == VAR_BIG) ? 32 : 64;
  const long long t1 = (g.r + bt - 1) / bt;
  const long long tiles = t1 * (t1 + 1) / 2 * g.count;
  long long want = (512 + tiles - 1) / tiles;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  long long kps = (rows + want - 1) / want;
  kps = (kps + 2 * bk - 1) / (2 * bk) * (2 * bk);
  gp.kps = (int)kps;
  gp.splitk = (int)((rows + kps - 1) / kps);
  // large-tile path: 128x128 tiles, lower triangle only
  const long long t2 = (g.r + 127) / 128;
  long long want2 = (768 + t2 * (t2 + 1) / 2 * g.count - 1) / (t2 * (t2 + 1) / 2 * g.count);
  if (want2 > 32) want2 = 32;
  if (want2 < 1) want2 = 1;
  gp.splitk2 = (int)want2;
  // 256 x 256 tiles: a single matrix (or a few) has fewer lower tiles than the GPU has compute units and is split over
  // the rows by up to 8; a batch that fills the GPU anyway is not
  const long long t3 = g.r / 256;
  gp.split_cap256 = (t3 * (t3 + 1) / 2 * g.count < 256) ? std::max(8, gp.splitk2) : gp.splitk2;
  return gp;
}

void plan_gram(Group& g) {
  g.gram_m = plan_gram_rows(g, g.m);
  g.gram_n = plan_gram_rows(g, g.n);
  // K1 (m x r output) and K2 (n x r output) on 128x128 tiles: split the contraction until about 512 workgroups exist
  g.k12_splitk = 1;
  g.direct12 = false;
  if (g.m % 256 == 0 && g.n % 256 == 0 && g.r % 128 == 0) {
    const long long tiles = std::min(g.m, g.n) / 128 * (g.r / 128) * g.count;
    const bool big_tiles = g.r % 256 == 0 && (std::min(g.m, g.n) / 256) * (g.r / 256) * g.count >= 128;
    if (!big_tiles && tiles < 512) g.k12_splitk = (int)std::min<long long>(8, (512 + tiles - 1) / tiles);
    g.direct12 = big_tiles && g.m * g.n * 2 < (1ll << 32);
  }
}

Carve carve_entry(const Group& g) {
  Carve c;
  memset(&c, 0, sizeof(c));
  size_t pos = 0;
  auto take = [&](int slot, size_t floats) {
    c.off[slot] = pos;
    pos += align_up(floats * sizeof(float), 256);
  };
  const size_t mr = (size_t)g.m * g.r, nr = (size_t)g.n * g.r, rr = (size_t)g.rp * g.rp;
  // buffers of the orthonormalisation are sized for the taller of the m x r (Dion step) and n x r (Lazy-Dion refresh) inputs
  const size_t xr = std::max(mr, nr);
  take(SLOT_Z, mr);
  take(SLOT_P1, xr);
  take(SLOT_P, mr);
  take(SLOT_R, nr);
  take(SLOT_C, rr);
  take(SLOT_L, rr);
  take(SLOT_W, rr);
  take(SLOT_T, rr);
  take(SLOT_CPART, rr * (size_t)std::max(std::max(std::max(g.gram_m.splitk, g.gram_m.splitk2), std::max(g.gram_n.splitk, g.gram_n.splitk2)),
                                         std::max(g.gram_m.split_cap256, g.gram_n.split_cap256)));
  take(SLOT_SPART, (size_t)((std::max(g.m, g.n) + COLNORM_CHUNK_MIN - 1) / COLNORM_CHUNK_MIN) * g.r);
  take(SLOT_S, g.r);
  take(SLOT_D, g.r);
  // bf16 operand copies (two bf16 values per float slot): only the large-tile bf16 kernels read them
  const size_t b = g.big ? 1 : 0;
  take(SLOT_QT16, b * ((nr + 1) / 2));
  take(SLOT_P16, b * ((xr + 1) / 2));
  take(SLOT_PT16, b * ((xr + 1) / 2));
  take(SLOT_R16, b * ((nr + 1) / 2));
  take(SLOT_Q16, b * ((nr + 1) / 2));
  take(SLOT_ZL16, b * ((xr + 1) / 2));
  take(SLOT_ZLT16, b * ((xr + 1) / 2));
  take(SLOT_WH16, b * (((size_t)g.r * g.r + 1) / 2));
  take(SLOT_WL16, b * (((size_t)g.r * g.r + 1) / 2));
  take(SLOT_EPART, GRAM_DEFECT_PARTS);
  take(SLOT_FAST, 1);
  // split-k partial results of K1 / K2: whole partial matrices off the direct-load path; on it (one matrix only) the
  // partial 256 x 256 tiles of a split last round, at most 256 of them
  take(SLOT_KPART, !g.big ? 0 : g.k12_splitk > 1 ? (size_t)g.k12_splitk * std::max(mr, nr) : (g.direct12 && g.count == 1) ? (size_t)256 * 256 * 256 : 0);
  take(SLOT_SYNC, 2 * (size_t)sync_words(g.rp / CHOL_NB));
  take(SLOT_B16, b * (((size_t)g.m * g.n + 1) / 2));
  take(SLOT_THR, g.rp);
  take(SLOT_NULL, g.rp);
  take(SLOT_GATE, 1);
  c.total = pos;
  return c;
}

bool shapes_ok(int count, const int64_t* m, const int64_t* n, const int64_t* r) {
  if (count < 0) return false;
  if (count > 0 && (!m || !n || !r)) return false;
  for (int i = 0; i < count; ++i) {
    if (m[i] <= 0 || n[i] <= 0 || r[i] <= 0) return false;
    if (r[i] > m[i] || r[i] > n[i]) return false;
    if (m[i] > 0x7fffff00LL || n[i] > 0x7fffff00LL) return false;
    if (r[i] > 32768) return false;
  }
  return true;
}

bool build_plan(int count, const int64_t* m, const int64_t* n, const int64_t* r, const int* form, int math,
                std::vector<Entry>& entries, std::vector<Group>& groups) {
  entries.resize(count);
  groups.clear();
  for (int i = 0; i < count; ++i) {
    int gi = -1;
    const int f = form ? form[i] : DION_FORM_STANDARD;
    for (size_t k = 0; k < groups.size(); ++k)
      if (groups[k].m == m[i] && groups[k].n == n[i] && groups[k].r == r[i] && groups[k].form == f) gi = (int)k;
    if (gi < 0) {
      Group g;
      memset(&g, 0, sizeof(g));
      g.m = m[i]; g.n = n[i]; g.r = r[i];
      g.form = f;
      g.rp = padded_rank(r[i]);
      g.big = math == DION_MATH_BF16 && g.m % 256 == 0 && g.n % 256 == 0 && g.r % 128 == 0;
      groups.push_back(g);
      gi = (int)groups.size() - 1;
    }
    entries[i].m = m[i]; entries[i].n = n[i]; entries[i].r = r[i];
    entries[i].form = f;
    entries[i].group = gi;
    groups[gi].count++;
  }
  int row = 0;
  for (auto& g : groups) {
    g.first_row = row;
    row += g.count;
    plan_gram(g);
    g.carve = carve_entry(g);
    g.bytes_per_entry = g.carve.total;
  }
  std::vector<int> next(groups.size());
  for (size_t k = 0; k < groups.size(); ++k) next[k] = groups[k].first_row;
  for (int i = 0; i < count; ++i) entries[i].row = next[entries[i].group]++;
  return true;
}

size_t header_bytes(int count) {   // pointer table, status words, step counter
  return align_up((size_t)count * NSLOTS * sizeof(void*), 256) + align_up((size_t)count * sizeof(int), 256) + 256;
}

}  // namespace

struct dion_state {
  int count, g_dtype, math;
  std::vector<Entry> entries;
  std::vector<Group> groups;
  char* ws;
  size_t ws_bytes;
  void** table;   // device, count * NSLOTS
  int* status;    // device, count ints (table-row order)
  unsigned long long* step_counter;   // device: number of steps enqueued so far (tags the flags of the Cholesky kernel)
  hipStream_t last_stream;
  bool timing;
  int cus;            // compute units of the device the state was created on
  bool force_panel;   // factor with a launch per panel even where the single-launch kernels would serve
  int orth_mode;
  unsigned chol_spin_limit;  // polls after which a wait inside that kernel gives up
  std::vector<hipEvent_t> events;      // groups * kEventsPerGroup
  // K1 on the direct-load path in parts (see stage_k1): a second stream for the parts of the bf16 copy, and events that
  // order them against the parts of the product.  Null when the state was made without them (the entry point that
  // allocates nothing): the copy then runs before the product, on the caller's stream.
  hipStream_t side_stream = nullptr;
  hipEvent_t ev_fork = nullptr, ev_part[K1_PARTS] = {}, ev_main[K1_PARTS] = {};
  std::vector<char> group_timed;       // which groups ran in the last call with timing on
};

#define HIPCHK(expr)                          \
  do {                                        \
    hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) return DION_ELAUNCH; \
  } while (0)

namespace {

void destroy_side_stream(dion_state* st) {
  if (st->ev_fork) (void)hipEventDestroy(st->ev_fork);
  for (int q = 0; q < K1_PARTS; ++q) {
    if (st->ev_part[q]) (void)hipEventDestroy(st->ev_part[q]);
    if (st->ev_main[q]) (void)hipEventDestroy(st->ev_main[q]);
    st->ev_part[q] = st->ev_main[q] = nullptr;
  }
  if (st->side_stream) (void)hipStreamDestroy(st->side_stream);
  st->ev_fork = nullptr;
  st->side_stream = nullptr;
}
// The second stream and its events (default priority; the stream does not synchronise with the legacy default stream,
// which may be the caller's).  On failure the state simply goes without them.
void create_side_stream(dion_state* st) {
  bool ok = hipStreamCreateWithFlags(&st->side_stream, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&st->ev_fork, hipEventDisableTiming) == hipSuccess;
  for (int q = 0; ok && q < K1_PARTS; ++q)
    ok = hipEventCreateWithFlags(&st->ev_part[q], hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&st->ev_main[q], hipEventDisableTiming) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    destroy_side_stream(st);
  }
}

// Host part of creating a state: the plan, the carving of the workspace and the host image of the pointer table
// (M_dev / Q_dev may be null: those two slots are refreshed by every step anyway).  Touches no device memory.
int plan_state(dion_state* st, int count, const int64_t* m, const int64_t* n, const int64_t* r, const int* form, int g_dtype,
               int math, void* workspace_dev, size_t workspace_bytes, void* const* M_dev, void* const* Q_dev,
               std::vector<void*>& host) {
  st->count = count; st->g_dtype = g_dtype; st->math = math;
  build_plan(count, m, n, r, form, math, st->entries, st->groups);
  st->ws = (char*)workspace_dev;
  st->ws_bytes = workspace_bytes;
  st->table = (void**)st->ws;
  st->status = (int*)(st->ws + align_up((size_t)count * NSLOTS * sizeof(void*), 256));
  st->step_counter = (unsigned long long*)((char*)st->status + align_up((size_t)count * sizeof(int), 256));
  st->last_stream = nullptr;
  st->timing = false;
  st->force_panel = false;
  st->cus = 0;
  {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&st->cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || st->cus < 1)
      return DION_ELAUNCH;
  }
  st->orth_mode = DION_ORTH_CHOLQR2;
  st->chol_spin_limit = 1u << 20;
  st->group_timed.assign(st->groups.size(), 0);
  host.assign((size_t)count * NSLOTS, nullptr);
  size_t pos = header_bytes(count);
  std::vector<size_t> group_base(st->groups.size());
  for (size_t k = 0; k < st->groups.size(); ++k) {
    group_base[k] = pos;
    st->groups[k].ws_off = pos;
    pos += st->groups[k].bytes_per_entry * st->groups[k].count;
  }
  for (int i = 0; i < count; ++i) {
    const Entry& e = st->entries[i];
    const Group& g = st->groups[e.group];
    const Carve c = carve_entry(g);
    char* base = st->ws + group_base[e.group] + (size_t)(e.row - g.first_row) * g.bytes_per_entry;
    void** rowp = &host[(size_t)e.row * NSLOTS];
    for (int sl = SLOT_Z; sl <= SLOT_D; ++sl) rowp[sl] = base + c.off[sl];
    for (int sl = SLOT_QT16; sl <= SLOT_GATE; ++sl) rowp[sl] = base + c.off[sl];
    rowp[SLOT_STATUS] = st->status + e.row;
    rowp[SLOT_M] = M_dev ? M_dev[i] : nullptr;
    rowp[SLOT_Q] = Q_dev ? Q_dev[i] : nullptr;
  }
  return DION_OK;
}

GemmArgs base_args(const dion_state* st, const Group& g) {
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.table = st->table + (size_t)g.first_row * NSLOTS;
  a.nslots = NSLOTS;
  a.splitk = 1;
  a.sub_count = 1;
  a.status_slot = -1;
  a.noop_slot = -1;
  a.E.colsq_slot = -1;
  a.side_slot = -1;
  a.tail_slot = -1;
  a.E.alpha = 1.f;
  return a;
}
GemmArgs rebase(GemmArgs a, int row_offset) {
  a.table = a.table + (size_t)row_offset * NSLOTS;
  return a;
}
Operand opnd(int slot0, long long off, long long ld, long long sub_stride = 0, int slot1 = 0) {
  Operand o;
  o.slot0 = slot0; o.slot1 = slot1; o.off = off; o.ld = ld; o.sub_stride = sub_stride;
  return o;
}

// Tile size and split over the rows of the Gram matrix of `batch` rows x r matrices on the split-bf16 path.
// 256 x 256 tiles (direct-load kernel) when the lower triangle of such tiles, split over the rows as far as the
// partial-result buffer allows, fills at least half of the GPU and every split still has a contraction worth
// starting a pipeline for; else 128 x 128 tiles with a deeper split.
// Split over the rows.  The plain choice: as many workgroups per tile as it takes to reach the number of compute
// units.  With s workgroups per tile the kernel runs in ceil(tiles s / 256) rounds of 1/s of the contraction each,
// and the partial results cost a pass over s of them afterwards (about 0.06 us per tile and partial): where that
// estimate finds a split at least a fifth cheaper (136 tiles at r = 4096: two per tile make a second round for 16
// workgroups, seven make four full rounds), it is taken; smaller predicted gains did not show up in measurements
// (r = 2048: seven per tile slower than six).  Every split must keep a contraction worth starting a pipeline for.
struct GramChoice {
  bool big;
  int split;
};
GramChoice choose_gram(const Group& g, int batch, long long rows, const GramPlan& gp) {
  const long long r = g.r;
  const long long t256 = r / 256, tiles256 = t256 * (t256 + 1) / 2 * batch;
  int big_split = 1;
  if (tiles256 > 0) {
    const double t_full = 3.0 * (double)(rows / 64) * 1.8, t_red = 0.06 * (double)tiles256;
    auto cost = [&](int sp) {
      const double rounds = (double)((tiles256 * sp + 255) / 256);
      return rounds / sp * t_full + (sp > 1 ? sp * t_red + 5.0 : 0.0);
    };
    big_split = (int)std::min<long long>(std::min(gp.splitk2, gp.split_cap256), (256 + tiles256 - 1) / tiles256);
    if (big_split < 1) big_split = 1;
    int best = big_split;
    for (int sp = 1; sp <= gp.split_cap256; ++sp) {
      if (sp > 1 && 3 * (rows / 64) / sp < 16) break;
      if (cost(sp) < cost(best)) best = sp;
    }
    if (cost(best) < 0.8 * cost(big_split)) big_split = best;
  }
  GramChoice c;
  c.big = r % 256 == 0 && rows % 64 == 0 && tiles256 * big_split >= 128 && 3 * (rows / 64) / big_split >= 16;
  c.split = big_split;
  return c;
}

// One Cholesky-QR pass (Appendix A): out = in * chol(in^T in)^-T, for `batch` matrices of `rows` x r starting at
// table row `row0` of group g (rows = m in a Dion step, n in a Lazy-Dion refresh; gp is the matching plan).
// With `split` the two large products run on the bf16 matrix pipe with split operands (x = hi + lo,
// three partial products), which carries about 16 mantissa bits at a fraction of the fp32 MFMA cost; the
// Cholesky factorisation and the triangular inverse stay in fp32.
// rank_tol > 0: the factorisation tolerates linearly dependent columns (see CholPanelPtrs::thr): they come out as zero
// columns of `out` and are marked in SLOT_NULL, instead of a breakdown.
// Where a split-bf16 pass finds the bf16 halves of its input (row-major, x = hi + lo) and whether its producer has
// already left them there; where its triangular multiply may leave the halves of its output for the next pass
// (-1: nowhere).  *wrote_out tells whether it did (only the direct-load core can).
struct SplitIO {
  int in_hi = SLOT_P16, in_lo = SLOT_ZL16;
  bool ready = false;
  int out_hi = -1, out_lo = -1;
  bool* wrote_out = nullptr;
};
int cholqr_pass(dion_state* st, const Group& g, int row0, int batch, long long rows, const GramPlan& gp, int slot_in,
                int slot_out, float piv_lo, float piv_hi, bool split, bool adaptive, float shift_rel, int pass, hipStream_t s,
                float rank_tol = 0.f, SplitIO io = SplitIO(), int gate_slot = -1) {
  if (io.wrote_out) *io.wrote_out = false;
  // gate_slot >= 0 (fp32 passes only): every launch of the pass leaves alone the matrices whose int32 there is non-zero
  if (gate_slot >= 0 && (split || adaptive || rank_tol > 0.f)) return DION_EINVAL;
  void* const* tab = st->table + (size_t)(g.first_row + row0) * NSLOTS;
  const int r = (int)g.r, rp = g.rp;
  const long long rr = (long long)rp * rp;
  GemmArgs base = rebase(base_args(st, g), row0);
  const int nb = rp / CHOL_NB;
  // Workgroups per matrix for the single-launch driver: all of a launch must be resident at once (one per compute
  // unit), so a batch shares the compute units this GPU has (read once, when the state was created).
  int spr = 0, spc = 0, chain = 0;
  if (!st->force_panel) plan_chol_grid(st->cus, batch, nb, &spr, &spc, &chain);
  const bool use_stream = spr > 0;
  // The split-K partial Gram matrices of an adaptive pass are added up by its defect kernel, which reads the whole
  // Gram matrix anyway (and stores the sum); other passes run a reduction kernel.  (Adding them up inside the
  // single-launch factorisation, every workgroup its own tiles, was measured slower than that kernel.)
  const bool sum_in_defect = adaptive && shift_rel == 0.f;
  int c_nsplit = 1;
  // Gram matrix (lower tiles), split over m when the tile count alone cannot fill the GPU
  if (split) {
    const GramChoice gc = choose_gram(g, batch, rows, gp);
    const bool gram_big = gc.big;
    const int big_split = gc.split;
    // On 256 x 256 tiles the Gram matrix reads the two row-major halves as operands stored with k (the row index) as
    // the slow index; the 128-wide-tile kernel needs transposed copies.  (An adaptive pass on the latter needs the low
    // part in row-major order only if it goes on to its product: made after the decision.)
    if (!gram_big && (io.in_hi != SLOT_P16 || io.in_lo != SLOT_ZL16 || io.ready)) return DION_EINVAL;   // (that kernel's copies go to fixed slots)
    if (!io.ready)
      HIPCHK(launch_split_bf16(tab, NSLOTS, batch, slot_in, r, rows, r, io.in_hi, (gram_big || !adaptive) ? io.in_lo : -1,
                               gram_big ? -1 : SLOT_PT16, gram_big ? -1 : SLOT_ZLT16, s));
    GemmArgs a = base;
    a.M = r; a.N = r; a.K = 3 * (int)rows;
    a.nseg = 3; a.kseg = (int)rows;
    const int hi = gram_big ? io.in_hi : SLOT_PT16, lo = gram_big ? io.in_lo : SLOT_ZLT16;
    a.segA[0] = hi; a.segB[0] = hi;
    a.segA[1] = hi; a.segB[1] = lo;
    a.segA[2] = lo; a.segB[2] = hi;
    a.A = opnd(hi, 0, gram_big ? r : rows);
    a.B = opnd(hi, 0, gram_big ? r : rows);
    a.lower_only = 1;
    const int gcfg = gram_big ? G2_256x256 : G2_128x128;
    a.splitk = gram_big ? big_split : gp.splitk2;
    // consecutive tiles of one split on one XCD: they share the rows of the split and many operand panels, so an
    // XCD's L2 fetches a fraction of what a round-robin placement makes it fetch
    a.xcd_remap = gram_big ? 1 : 0;
    const int eff = gemm2_nt_splitk(gcfg, a);
    a.E.slot = (eff > 1) ? SLOT_CPART : SLOT_C;
    a.E.ld = rp;
    a.E.split_stride = rr;
    HIPCHK(gemm2_nt(gcfg, a, batch, s, gram_big ? (KS_A | KS_B) : 0));
    c_nsplit = eff;
  } else {
    GemmArgs a = base;
    a.M = r; a.N = r; a.K = (int)rows;
    a.A = opnd(slot_in, 0, r);
    a.B = opnd(slot_in, 0, r);
    a.lower_only = 1;
    a.splitk = gp.splitk;
    a.k_per_split = gp.kps;
    a.E.slot = (gp.splitk > 1) ? SLOT_CPART : SLOT_C;
    a.E.ld = rp;
    a.E.split_stride = rr;
    a.status_slot = gate_slot;
    HIPCHK(gemm_f32_tn(gp.variant, a, batch, s));
    c_nsplit = gp.splitk;
  }
  if (c_nsplit > 1 && !sum_in_defect) {
    HIPCHK(launch_reduce_partials(tab, NSLOTS, batch, SLOT_CPART, SLOT_C, r, rp, c_nsplit, rr, s, gate_slot));
    c_nsplit = 1;
  }
  if (shift_rel > 0.f) HIPCHK(launch_shift_diagonal(tab, NSLOTS, batch, r, rp, shift_rel, s, gate_slot));
  HIPCHK(launch_pad_identity(tab, NSLOTS, batch, SLOT_C, r, rp, s, gate_slot));
  if (rank_tol > 0.f) HIPCHK(launch_rank_threshold(tab, NSLOTS, batch, rp, rank_tol, s));
  // (W needs no clearing: its part above the block diagonal was zeroed at init and nothing ever writes there; the
  // rest is overwritten in full by the factorisation kernels, the merges below or the first-order factor)
  // Second pass: the input is already orthonormal to about 1e-5, so its Gram matrix is I + E with tiny E
  // and chol(I + E)^-1 = I - Phi(E) + O(E^2): no factorisation needed.  The decision is taken on the device
  // (||E||_F <= 1e-3, i.e. a second-order error below 1e-6); when it fails, the launches below do the full
  // factorisation, otherwise they return at once.
  const int skip = adaptive ? SLOT_FAST : gate_slot;
  if (adaptive) {
    // (bf16 mode: decision only, see the product at the end)
    HIPCHK(launch_first_order_inverse(tab, NSLOTS, batch, r, rp, 1e-3f, split, c_nsplit, rr, s));
    c_nsplit = 1;
  }
  base.status_slot = skip;
  // blocked right-looking Cholesky, one fused launch per 64-wide panel.  The kernel gets the addresses of
  // its buffers as arguments: a look-up in the pointer table would cost it one more memory round trip.
  CholPanelPtrs pp;
  {
    char* e0 = st->ws + g.ws_off + (size_t)row0 * g.bytes_per_entry;
    pp.C = (float*)(e0 + g.carve.off[SLOT_C]);
    pp.L = (float*)(e0 + g.carve.off[SLOT_L]);
    pp.W = (float*)(e0 + g.carve.off[SLOT_W]);
    pp.skip = skip >= 0 ? (const int*)(e0 + g.carve.off[skip]) : nullptr;
    pp.stride = (long long)(g.bytes_per_entry / sizeof(float));
    pp.status = st->status + g.first_row + row0;
    pp.thr = rank_tol > 0.f ? (const float*)(e0 + g.carve.off[SLOT_THR]) : nullptr;
    pp.nullmask = rank_tol > 0.f ? (int*)(e0 + g.carve.off[SLOT_NULL]) : nullptr;
  }
  bool fused_inverse = false;
  if (use_stream) {
    // the whole factorisation in one launch of at most 256 co-resident workgroups
    CholStreamArgs ca;
    ca.C = pp.C; ca.L = pp.L; ca.W = pp.W; ca.status = pp.status; ca.skip = pp.skip;
    ca.sync = (unsigned long long*)(st->ws + g.ws_off + (size_t)row0 * g.bytes_per_entry + g.carve.off[SLOT_SYNC]);
    ca.stride = pp.stride;
    ca.sync_stride = (long long)(g.bytes_per_entry / sizeof(unsigned long long));
    ca.rp = rp;
    ca.pr = spr; ca.pc = spc;
    ca.piv_lo = piv_lo; ca.piv_hi = piv_hi;
    ca.step_counter = st->step_counter;
    ca.pass = pass;
    ca.spin_limit = st->chol_spin_limit;
    ca.thr = pp.thr; ca.nullmask = pp.nullmask;
    ca.chain = chain;
    // with the chain in a workgroup of its own and up to 64 panels the helpers form W = L^-1 behind the factorisation
    fused_inverse = chain && nb <= FUSED_INV_MAX_NB && rank_tol <= 0.f;
    ca.vflag_off = fused_inverse ? fused_inv_flag_offset(nb) : 0;
    HIPCHK(launch_chol_stream(ca, batch, s));
  } else {
    for (int k = 0; k < rp; k += CHOL_NB)
      HIPCHK(launch_chol_panel(pp, batch, k, rp, piv_lo, piv_hi, s));
  }
  // W = L^-1 by merging neighbouring diagonal blocks: [[A,0],[C,D]]^-1 = [[A^-1,0],[-D^-1 C A^-1, D^-1]].
  // Blocks start as the 64-wide inverses left by the factorisation.
  if (fused_inverse) {
    // (done by the factorisation kernel)
  } else if (use_stream) {
    // all levels in one launch, by the same number of co-resident workgroups as the factorisation had
    InvTreeArgs ta;
    char* e0 = st->ws + g.ws_off + (size_t)row0 * g.bytes_per_entry;
    ta.L = pp.L; ta.W = pp.W; ta.T = (float*)(e0 + g.carve.off[SLOT_T]);
    ta.status = pp.status; ta.skip = pp.skip;
    ta.sync = (unsigned long long*)(e0 + g.carve.off[SLOT_SYNC]) + chol_sync_words(nb);
    ta.stride = pp.stride;
    ta.sync_stride = (long long)(g.bytes_per_entry / sizeof(unsigned long long));
    ta.rp = rp;
    ta.step_counter = st->step_counter;
    ta.pass = pass;
    ta.spin_limit = st->chol_spin_limit;
    HIPCHK(launch_inv_tree(ta, spr * spc + chain, batch, st->cus, s));
  } else {
    // one launch per product: an odd block is carried to the next level, so any multiple of 64 works; runs of equal,
    // evenly spaced pairs go out as one launch
    struct Blk { int off, size; };
    static_assert(32768 / CHOL_NB <= 512, "block list size");
    Blk cur[512], nxt[512];
    int ncur = 0;
    for (int o = 0; o < rp; o += CHOL_NB) cur[ncur++] = Blk{o, CHOL_NB};
    while (ncur > 1) {
      int nn = 0, i = 0;
      while (i + 1 < ncur) {
        const int sa = cur[i].size, sd = cur[i + 1].size, o = cur[i].off;
        int pairs = 0, j = i;
        while (j + 1 < ncur && cur[j].size == sa && cur[j + 1].size == sd && cur[j].off == o + pairs * (sa + sd)) {
          nxt[nn++] = Blk{cur[j].off, sa + sd};
          ++pairs;
          j += 2;
        }
        const long long stride = (long long)(sa + sd) * (rp + 1);
        const long long o11 = (long long)o * rp + o, o21 = (long long)(o + sa) * rp + o, o22 = (long long)(o + sa) * rp + (o + sa);
        {
          GemmArgs a = base;  // T = L21 W11
          a.M = sd; a.N = sa; a.K = sa; a.sub_count = pairs;
          a.A = opnd(SLOT_L, o21, rp, stride);
          a.B = opnd(SLOT_W, o11, rp, stride);
          a.E.slot = SLOT_T; a.E.off = o21; a.E.ld = rp; a.E.sub_stride = stride;
          HIPCHK(gemm_f32_nn(pick_variant(a.M, a.N, a.K, (long long)batch * pairs, true), a, batch, s));
        }
        {
          GemmArgs a = base;  // W21 = -W22 T
          a.M = sd; a.N = sa; a.K = sd; a.sub_count = pairs;
          a.A = opnd(SLOT_W, o22, rp, stride);
          a.B = opnd(SLOT_T, o21, rp, stride);
          a.E.slot = SLOT_W; a.E.off = o21; a.E.ld = rp; a.E.sub_stride = stride;
          a.E.alpha = -1.f;
          HIPCHK(gemm_f32_nn(pick_variant(a.M, a.N, a.K, (long long)batch * pairs, true), a, batch, s));
        }
        i = j;
      }
      if (i < ncur) nxt[nn++] = cur[i];
      for (int k = 0; k < nn; ++k) cur[k] = nxt[k];
      ncur = nn;
    }
  }
  base.status_slot = -1;
  if (split) {
    // (Adaptive pass whose input was found orthonormal to 1e-3: the input is the result.  Both consumers of it round
    // it to bf16, whose unit roundoff is 2e-3 per entry, so not even the first-order correction in - in Phi^T, itself
    // below 1e-3, would survive.  Such a pass runs in place, slot_out == slot_in: the product reads the bf16 copies
    // of its input, never the fp32 original, so it may overwrite that; and when the flag is set it has nothing to do.)
    HIPCHK(launch_split_bf16(tab, NSLOTS, batch, SLOT_W, rp, r, r, SLOT_WH16, SLOT_WL16, -1, -1, s, skip));
    if (adaptive && !choose_gram(g, batch, rows, gp).big)
      HIPCHK(launch_split_bf16(tab, NSLOTS, batch, slot_in, r, rows, r, -1, SLOT_ZL16, -1, -1, s, skip));
    GemmArgs a = base;  // out = in W^T with in = hi + lo, W = Wh + Wl
    if (adaptive) {
      if (slot_out != slot_in) return DION_EINVAL;
      a.noop_slot = SLOT_FAST;
    }
    a.M = (int)rows; a.N = r; a.K = 3 * r;
    a.nseg = 3; a.kseg = r;
    a.segA[0] = io.in_hi; a.segB[0] = SLOT_WH16;
    a.segA[1] = io.in_hi; a.segB[1] = SLOT_WL16;
    a.segA[2] = io.in_lo; a.segB[2] = SLOT_WH16;
    a.A = opnd(io.in_hi, 0, r);
    a.B = opnd(SLOT_WH16, 0, r);
    a.tri_k = 1;
    a.E.slot = slot_out; a.E.ld = r;
    a.xcd_remap = 1;
    int cfg = (rows % 256 == 0 && r % 256 == 0 && (rows / 256) * (r / 256) * batch >= 128) ? G2_256x256 : G2_128x128;
    // One matrix whose 256-wide tiles make a single round of workgroups: the triangular factor makes the last
    // column tile cost r / 256 times the first, and that one sets the time.  128-wide column tiles give two
    // rounds, costliest first.
    if (cfg == G2_256x256 && batch == 1 && (rows / 256) * (r / 256) <= 256 && (rows / 256) % 8 == 0) {
      cfg = G2_256x128;
      a.heavy_first = 1;
    } else if (cfg == G2_256x256 && batch == 1 && (rows / 256) % 8 == 0) {
      a.heavy_first = 1;   // several rounds of 256-wide tiles: still the costliest columns first, so that the cheap ones fill the tail
    }
    if (io.out_hi >= 0 && gemm2_nt_is_direct(cfg, a)) {
      // the halves of the result, for the pass that follows (other buffers than this pass' input: other workgroups
      // still read that)
      if (io.out_hi == io.in_hi || io.out_lo == io.in_lo) return DION_EINVAL;
      a.E.split_hi1 = io.out_hi + 1;
      a.E.split_lo1 = io.out_lo + 1;
      if (io.wrote_out) *io.wrote_out = true;
    }
    HIPCHK(gemm2_nt(cfg, a, batch, s));
  } else {
    GemmArgs a = base;  // out = in W^T   (= in L^-T)
    a.M = (int)rows; a.N = r; a.K = r;
    a.A = opnd(slot_in, 0, r);
    a.B = opnd(SLOT_W, 0, rp);
    a.E.slot = slot_out; a.E.ld = r;
    a.xcd_remap = 1;
    a.status_slot = gate_slot;
    HIPCHK(gemm_f32_nt(pick_variant(a.M, a.N, a.K, batch, true), a, batch, s));
  }
  return DION_OK;
}

// What the stages of a step share: the matrices [row0, row0 + batch) of one shape group.
struct RowCtx {
  dion_state* st;
  const Group* g;
  int gi, row0, batch;
  void* const* tab;
  bool bf16, gbf16;
  bool big;   // large-tile bf16 kernels: need tile-aligned shapes and bf16 copies of the small operands
  GemmArgs base;
  hipEvent_t* ev;   // start / end event per stage, or nullptr
  hipStream_t s;
};

RowCtx make_ctx(dion_state* st, int gi, int row0, int batch, hipStream_t s) {
  RowCtx c;
  c.st = st; c.g = &st->groups[gi]; c.gi = gi; c.row0 = row0; c.batch = batch; c.s = s;
  c.tab = st->table + (size_t)(c.g->first_row + row0) * NSLOTS;
  c.bf16 = st->math == DION_MATH_BF16;
  c.gbf16 = st->g_dtype == DION_G_BF16;
  c.big = c.g->big;
  c.base = rebase(base_args(st, *c.g), row0);
  c.ev = st->timing ? &st->events[(size_t)gi * kEventsPerGroup] : nullptr;
  return c;
}
int mark(const RowCtx& c, int stage, int end) {
  if (c.ev) HIPCHK(hipEventRecord(c.ev[2 * stage + end], c.s));
  return DION_OK;
}
int tile_cfg2(const RowCtx& c, long long Mo, long long No) {
  return (Mo % 256 == 0 && No % 256 == 0 && (Mo / 256) * (No / 256) * c.batch >= 128) ? G2_256x256 : G2_128x128;
}

// Direct-load path of K1 and K2: both read the same row-major bf16 copy of M + G from memory.  For K1 its contraction
// index is the fast one; K2 contracts over its rows and takes it with k as the slow index (transposing LDS reads), as
// both products take their r-column operands (Q, P) in their own row-major order.  Taken when the plan has the buffer
// and this call's batch still fills the GPU with 256 x 256 tiles.
// Tile order of these two products: column groups of four 256-wide tile columns (all row tiles of a group before the
// next group).  The 32 tiles that run at one time on an XCD then form about 8 x 4 tiles instead of 2 x 16 at r = 4096,
// two thirds of the operand panels: K2 at 16384 x 53248 r = 4096 7.2 -> 6.1 ms, K1 1 %; r <= 1024 has no more than four
// tile columns anyway.
constexpr int kDirect12GroupN = 4;
bool direct12(const RowCtx& c) {
  const Group& g = *c.g;
  return c.big && g.direct12 && tile_cfg2(c, g.m, g.r) == G2_256x256 && tile_cfg2(c, g.n, g.r) == G2_256x256;
}
// The bf16 copy of M + G for the K1 / K2 of this call (a no-op off the direct-load path).
int stage_b16(const RowCtx& c) {
  if (!direct12(c)) return DION_OK;
  HIPCHK(launch_sum_bf16(c.tab, NSLOTS, c.batch, SLOT_M, SLOT_G, c.gbf16, SLOT_B16, c.g->m, c.g->n, c.s));
  return DION_OK;
}

// K1: Z = (M+G) Q with Q (n x r, fp32) taken from slot_q.  keep_b16: the large-tile kernel also leaves bf16(M+G) in
// SLOT_B16 for a K2 that follows.
// split_out: on the direct-load path, also leave the result's bf16 halves in (SLOT_PT16, SLOT_ZLT16) for an
// orthonormalisation that follows (*split_done tells whether that happened).
// b16_in_parts: bf16(M+G) has not been made yet (direct-load path, k1_in_parts(c) holds): it is made here, in K1_PARTS
// column blocks on the state's second stream, and the product contracts over block q once it is there, adding to what
// the blocks before it gave.  A streaming pass and a product running side by side take less than one after the other
// (the product leaves the memory system idle, the pass leaves the matrix cores idle), and started in this order -
// each part of the pass only once the product before it is on its way - the product's workgroups get their compute
// units first and the pass fills in.  Everything on the second stream is back on the caller's before the last part of
// the product starts; a caller capturing its stream into a graph captures both.
// Parts over blocks of rows instead (K1_ROW_PARTS): each part a product of its own over a block of rows of M + G, whole
// rounds of tiles each, nothing to add up and nothing read back - possible where a quarter of the output still has
// a multiple of the compute units' number of tiles (16384 x 53248 at r = 4096: 4 x 256), and then the better choice
// (there the parts over the contraction gained nothing: they reread and rewrite a 268 MB result three times).
enum { K1_WHOLE = 0, K1_K_PARTS = 1, K1_ROW_PARTS = 2 };
bool k1_in_parts(const RowCtx& c);
int k1_parts_mode(const RowCtx& c) {
  const Group& g = *c.g;
  if (direct12(c) && c.st->side_stream && (g.m / 256) % K1_PARTS == 0) {
    const long long tiles = (g.m / 256 / K1_PARTS) * (g.r / 256);   // (per matrix, as below: alone and in a batch alike)
    const double hidden = 0.35 * (8.0 * (double)g.m * (double)g.n / 5.2e12);
    if (tiles % c.st->cus == 0 && hidden > 1.25 * (K1_PARTS - 1) * 50e-6) return K1_ROW_PARTS;
  }
  return k1_in_parts(c) ? K1_K_PARTS : K1_WHOLE;
}
bool k1_in_parts(const RowCtx& c) {
  const Group& g = *c.g;
  if (!direct12(c) || !c.st->side_stream) return false;
  if ((g.n / 64) % K1_PARTS || (g.n / K1_PARTS) % 8) return false;
  // (a single matrix whose tiles leave a short last round has that round split over k, which a part of a contraction
  // does not do)
  const long long tiles = (g.m / 256) * (g.r / 256) * c.batch;
  if (!(c.batch > 1 || tiles % c.st->cus == 0 || tiles < c.st->cus)) return false;
  // Worth it?  Side by side, the pass and the product took 0.65 of what they take one after the other as long as
  // neither outlasts the other (measured at 16384 x 53248, r = 1024: 2.85 -> 2.45 ms for the stage), and every part
  // after the first reads and rewrites the m x r result and ramps up and down once more (about 50 us).  At r = 4096
  // the two balance (7.26 against 7.33 ms); with short contractions (8192 x 8192, or the 196 matrices of the 3B
  // model) the parts cost far more than they hide.
  // (Judged per matrix, whatever the batch: a matrix is then stepped with the same arithmetic alone and in a batch.)
  const double hidden = 0.35 * (8.0 * (double)g.m * (double)g.n / 5.2e12);
  const double extra = (K1_PARTS - 1) * (8.0 * (double)g.m * (double)g.r / 5.0e12 + 50e-6);
  return hidden > 1.25 * extra;
}
int stage_k1(const RowCtx& c, bool keep_b16, int slot_q = SLOT_Q, bool split_out = false, bool* split_done = nullptr,
             int b16_in_parts = K1_WHOLE) {
  if (split_done) *split_done = false;
  const Group& g = *c.g;
  const int m = (int)g.m, n = (int)g.n, r = (int)g.r;
  GemmArgs a = c.base;
  a.M = m; a.N = r; a.K = n;
  a.A = opnd(SLOT_M, 0, n, 0, SLOT_G);
  a.E.slot = SLOT_Z; a.E.ld = r;
  a.xcd_remap = 1;
  if (c.big) {
    if (direct12(c)) {
      dion_state* st = c.st;
      if (b16_in_parts) {
        if (k1_parts_mode(c) != b16_in_parts) return DION_EINVAL;
        HIPCHK(hipEventRecord(st->ev_fork, c.s));
        HIPCHK(hipStreamWaitEvent(st->side_stream, st->ev_fork, 0));
      }
      // Q as bf16 in its own row-major order (n x r): the right operand with k, its row index, as the slow index
      HIPCHK(launch_convert_bf16(c.tab, NSLOTS, c.batch, slot_q, SLOT_QT16, -1, n, r, c.s));
      a.B = opnd(SLOT_QT16, 0, r);
      a.A = opnd(SLOT_B16, 0, n);
      a.group_n = kDirect12GroupN;
      if (g.count == 1) { a.cus = c.st->cus; a.tail_slot = SLOT_KPART; }   // a short last round is split over k
      if (split_out) {
        a.E.split_hi1 = SLOT_PT16 + 1;
        a.E.split_lo1 = SLOT_ZLT16 + 1;
        if (split_done) *split_done = true;
      }
      if (!b16_in_parts) {
        HIPCHK(gemm2_nt(G2_256x256, a, c.batch, c.s, KS_B));
        return DION_OK;
      }
      if (b16_in_parts == K1_ROW_PARTS) {
        const long long rows = m / K1_PARTS;
        for (int q = 0; q < K1_PARTS; ++q) {
          if (q >= 1) HIPCHK(hipStreamWaitEvent(st->side_stream, st->ev_main[q - 1], 0));
          HIPCHK(launch_sum_bf16_cols(c.tab, NSLOTS, c.batch, SLOT_M, SLOT_G, c.gbf16, SLOT_B16, m, n, q * rows, rows, 0, n, st->side_stream));
          HIPCHK(hipEventRecord(st->ev_part[q], st->side_stream));
          HIPCHK(hipStreamWaitEvent(c.s, st->ev_part[q], 0));
          HIPCHK(hipEventRecord(st->ev_main[q], c.s));
          GemmArgs ap = a;
          ap.M = (int)rows;
          ap.A.off = q * rows * n;
          ap.E.off = q * rows * r;
          HIPCHK(gemm2_nt(G2_256x256, ap, c.batch, c.s, KS_B));
        }
        return DION_OK;
      }
      // (equal parts: unequal ones, a short first part of the copy or a short last part of the product, measured the same)
      const long long cols = n / K1_PARTS;
      for (int q = 0; q < K1_PARTS; ++q) {
        if (q >= 1) HIPCHK(hipStreamWaitEvent(st->side_stream, st->ev_main[q - 1], 0));
        HIPCHK(launch_sum_bf16_cols(c.tab, NSLOTS, c.batch, SLOT_M, SLOT_G, c.gbf16, SLOT_B16, m, n, 0, m, q * cols, cols, st->side_stream));
        HIPCHK(hipEventRecord(st->ev_part[q], st->side_stream));
        HIPCHK(hipStreamWaitEvent(c.s, st->ev_part[q], 0));
        HIPCHK(hipEventRecord(st->ev_main[q], c.s));
        GemmArgs ap = a;
        ap.slab_first = q * (int)(cols / 64);
        ap.slab_count = (int)(cols / 64);
        ap.E.beta = q ? 1.f : 0.f;
        if (q + 1 < K1_PARTS) { ap.E.split_hi1 = 0; ap.E.split_lo1 = 0; }   // the halves of the result come from its last part
        HIPCHK(gemm2_nt(G2_256x256, ap, c.batch, c.s, KS_B));
      }
      return DION_OK;
    }
    HIPCHK(launch_convert_bf16(c.tab, NSLOTS, c.batch, slot_q, -1, SLOT_QT16, n, r, c.s));
    a.B = opnd(SLOT_QT16, 0, n);
    if (keep_b16) a.side_slot = SLOT_B16;
    const int c1 = tile_cfg2(c, m, r);
    if (c1 == G2_128x128 && g.k12_splitk > 1) {
      a.splitk = g.k12_splitk; a.E.slot = SLOT_KPART; a.E.split_stride = (long long)m * r;
      const int eff = gemm2_k1_splitk(c1, a);
      HIPCHK(gemm2_k1(c1, c.gbf16, a, c.batch, c.s));
      HIPCHK(launch_sum_partials(c.tab, NSLOTS, c.batch, SLOT_KPART, SLOT_Z, (long long)m * r, eff, c.s));
    } else {
      HIPCHK(gemm2_k1(c1, c.gbf16, a, c.batch, c.s));
    }
  } else {
    a.B = opnd(slot_q, 0, r);
    HIPCHK(gemm_k1(pick_variant(m, r, n, c.batch, true), c.bf16, c.gbf16, a, c.batch, c.s));
  }
  return DION_OK;
}

// K2: R = (M+G)^T P with P (m x r) in slot_p (fp32) and, on the large-tile paths, a bf16 copy of it: row-major in
// SLOT_P16 for the direct-load path, transposed in SLOT_PT16 for the 128-wide-tile kernel.
// from_b16: a K1 of this step has left bf16(M+G) in SLOT_B16 (large-tile path only).
// colsq_chunks: if given, the product may leave per-column partial sums of squares of R in SLOT_SPART (it does on the
// direct-load path); *colsq_chunks then is their number of chunks, else 0.
int stage_k2(const RowCtx& c, int slot_p, bool from_b16 = true, int* colsq_chunks = nullptr) {
  const Group& g = *c.g;
  const int m = (int)g.m, n = (int)g.n, r = (int)g.r;
  if (colsq_chunks) *colsq_chunks = 0;
  GemmArgs a = c.base;
  a.M = n; a.N = r; a.K = m;
  a.A = opnd(SLOT_M, 0, n, 0, SLOT_G);
  a.E.slot = SLOT_R; a.E.ld = r;
  a.xcd_remap = 1;
  if (c.big) {
    // M + G was rounded to bf16 once, by K1, and is read back from there (2 bytes per element instead of 6)
    a.B = opnd(SLOT_PT16, 0, m);
    if (direct12(c)) {
      // both operands with k (the row index of M + G and of P) as the slow index: bf16(M + G) as K1 reads it, and the
      // row-major bf16 copy of P
      a.A = opnd(SLOT_B16, 0, n);
      a.B = opnd(SLOT_P16, 0, r);
      a.group_n = kDirect12GroupN;
      if (g.count == 1) { a.cus = c.st->cus; a.tail_slot = SLOT_KPART; }   // a short last round is split over k
      if (colsq_chunks) {
        *colsq_chunks = gemm2_nt_colsq_chunks(G2_256x256, a, KS_A | KS_B);
        if (*colsq_chunks > 0) a.E.colsq_slot = SLOT_SPART;
      }
      HIPCHK(gemm2_nt(G2_256x256, a, c.batch, c.s, KS_A | KS_B));
      return DION_OK;
    }
    if (from_b16) a.A = opnd(SLOT_B16, 0, n);
    const int c2 = tile_cfg2(c, n, r);
    if (c2 == G2_128x128 && g.k12_splitk > 1) {
      a.splitk = g.k12_splitk; a.E.slot = SLOT_KPART; a.E.split_stride = (long long)n * r;
      const int eff = gemm2_k2_splitk(c2, a);
      HIPCHK(gemm2_k2(c2, c.gbf16, a, c.batch, c.s, from_b16));
      HIPCHK(launch_sum_partials(c.tab, NSLOTS, c.batch, SLOT_KPART, SLOT_R, (long long)n * r, eff, c.s));
    } else {
      HIPCHK(gemm2_k2(c2, c.gbf16, a, c.batch, c.s, from_b16));
    }
  } else {
    a.B = opnd(slot_p, 0, r);
    HIPCHK(gemm_k2(pick_variant(n, r, m, c.batch, true), c.bf16, c.gbf16, a, c.batch, c.s));
  }
  return DION_OK;
}

// Orthonormalisation of the rows x r matrices in slot_a; slot_b is a second buffer of that size.  The result
// ends up in slot_final (CholeskyQR2: a -> b -> final, so final may be a; shifted CholeskyQR3: a -> b -> a ->
// final, so final must not be a).  On the split-bf16 path the products read bf16 copies of their input, never the
// fp32 original, so a pass may write where it reads: the first pass already writes to slot_final and the last,
// adaptive one runs there in place, which leaves it nothing to do when it finds its input orthonormal enough.
// True when the orthonormalisation of these rows x r matrices runs as plain CholeskyQR2 on the split-bf16 path with the
// Gram matrix on 256 x 256 tiles: then the halves of a pass' input may come from the epilogue of whatever produced it.
bool orth_fuses(const RowCtx& c, long long rows, const GramPlan& gp, float rank_tol) {
  return c.big && rank_tol == 0.f && c.st->orth_mode != DION_ORTH_SHIFTED_CHOLQR3 && choose_gram(*c.g, c.batch, rows, gp).big;
}
// rank_tol > 0: CholeskyQR2 that tolerates linearly dependent columns (zero columns of the result, marked in SLOT_NULL).
// in_split_ready: the producer of slot_a has left its bf16 halves in (SLOT_PT16, SLOT_ZLT16), row-major (see orth_fuses).
int stage_orth_plain(const RowCtx& c, long long rows, const GramPlan& gp, int slot_a, int slot_b, int slot_final, float rank_tol,
                     bool in_split_ready);
// With DION_ORTH_CHOLQR2_FALLBACK (and three distinct buffers, slot_a left intact by the plain passes): after the plain
// passes a small kernel looks at the status words; for the matrices that report a numerical breakdown it clears the
// word and opens the gate of three more passes, which are enqueued in any case and return at once for everybody else:
// shifted CholeskyQR3 in fp32 arithmetic from the untouched input (a -> b -> a -> final), whatever the state's
// arithmetic mode, since the split-bf16 products carry 16 bits and a Gram matrix squares the condition number.
// A matrix that these passes cannot factor either (exact rank deficiency) gets its breakdown status back from them.
int stage_orth(const RowCtx& c, long long rows, const GramPlan& gp, int slot_a, int slot_b, int slot_final, float rank_tol = 0.f,
               bool in_split_ready = false) {
  int rc = stage_orth_plain(c, rows, gp, slot_a, slot_b, slot_final, rank_tol, in_split_ready);
  if (rc != DION_OK || c.st->orth_mode != DION_ORTH_CHOLQR2_FALLBACK || rank_tol > 0.f) return rc;
  if (slot_final == slot_a || slot_final == slot_b || slot_a == slot_b) return DION_OK;   // (callers without a third buffer: plain)
  dion_state* st = c.st;
  const Group& g = *c.g;
  HIPCHK(launch_fallback_decide(c.tab, NSLOTS, c.batch, c.s));
  SplitIO none;
  rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_a, slot_b, 0.f, 3.0e38f, false, false, 1e-5f, 4, c.s, 0.f, none, SLOT_GATE);
  if (rc != DION_OK) return rc;
  // (the shifted pass leaves singular values sigma_j / sqrt(sigma_j^2 + shift): a pivot below 1e-6 here means a
  // condition number beyond 1e5 or a rank-deficient input, whose pivot is rounding noise of either sign)
  rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_b, slot_a, 1e-6f, 3.0e38f, false, false, 0.f, 5, c.s, 0.f, none, SLOT_GATE);
  if (rc != DION_OK) return rc;
  return cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_a, slot_final, 0.1f, 10.f, false, false, 0.f, 6, c.s, 0.f, none, SLOT_GATE);
}
int stage_orth_plain(const RowCtx& c, long long rows, const GramPlan& gp, int slot_a, int slot_b, int slot_final, float rank_tol,
                     bool in_split_ready) {
  dion_state* st = c.st;
  const Group& g = *c.g;
  const bool in_place = c.big;
  int rc;
  if (rank_tol > 0.f) {
    // Three passes.  Every column's pivot is measured against that column's own squared norm; columns that the first
    // pass drops come out exactly zero, meet a zero threshold and a zero pivot in the later passes, and are dropped
    // again.  The columns that stay can be badly conditioned among themselves (condition numbers of a few thousand
    // while the buffer is still filling up), which is more than two passes repair: the second pass brings the
    // first one's result to within the reach of the third, whose pivots are checked as usual.
    const int mid = in_place ? slot_final : slot_a;
    rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_a, slot_b, 0.f, 3.0e38f, c.big, false, 0.f, 1, c.s, rank_tol);
    if (rc != DION_OK) return rc;
    rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_b, mid, 0.f, 3.0e38f, c.big, false, 0.f, 2, c.s, rank_tol);
    if (rc != DION_OK) return rc;
    return cholqr_pass(st, g, c.row0, c.batch, rows, gp, mid, slot_final, 0.1f, 10.f, c.big, true, 0.f, 3, c.s, rank_tol);
  }
  // first pass: any positive finite pivot; last pass: the Gram matrix of a nearly orthonormal input has pivots near 1
  if (st->orth_mode == DION_ORTH_SHIFTED_CHOLQR3) {
    // Shifted Cholesky-QR first (the Gram matrix plus a small multiple of its trace cannot break down and
    // leaves a factor with a condition number of a few hundred), then CholeskyQR2 on that.  The product of
    // the three triangular factors is still the QR factor.
    const int mid = in_place ? slot_final : slot_a;
    rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_a, slot_b, 0.f, 3.0e38f, c.big, false, 1e-5f, 1, c.s);
    if (rc != DION_OK) return rc;
    rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_b, mid, 0.f, 3.0e38f, c.big, false, 0.f, 2, c.s);
    if (rc != DION_OK) return rc;
    return cholqr_pass(st, g, c.row0, c.batch, rows, gp, mid, slot_final, 0.1f, 10.f, c.big, true, 0.f, 3, c.s);
  }
  const int mid = in_place ? slot_final : slot_b;
  if (orth_fuses(c, rows, gp, rank_tol)) {
    // Both passes read row-major halves (the Gram matrix takes them with k as the slow index), so nothing has to be
    // transposed and the two transposed-copy buffers are free: the first pass takes its input's halves from there
    // (left by the product that made the input, or by the split kernel) and its triangular multiply leaves the halves
    // of its result where the second pass, and in the end the consumers of P, look for them.
    bool wrote = false;
    SplitIO io1;
    io1.in_hi = SLOT_PT16; io1.in_lo = SLOT_ZLT16; io1.ready = in_split_ready;
    io1.out_hi = SLOT_P16; io1.out_lo = SLOT_ZL16; io1.wrote_out = &wrote;
    rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_a, mid, 0.f, 3.0e38f, c.big, false, 0.f, 1, c.s, 0.f, io1);
    if (rc != DION_OK) return rc;
    SplitIO io2;
    io2.ready = wrote;
    return cholqr_pass(st, g, c.row0, c.batch, rows, gp, mid, slot_final, 0.1f, 10.f, c.big, true, 0.f, 2, c.s, 0.f, io2);
  }
  if (in_split_ready) return DION_EINVAL;
  rc = cholqr_pass(st, g, c.row0, c.batch, rows, gp, slot_a, mid, 0.f, 3.0e38f, c.big, false, 0.f, 1, c.s);
  if (rc != DION_OK) return rc;
  return cholqr_pass(st, g, c.row0, c.batch, rows, gp, mid, slot_final, 0.1f, 10.f, c.big, true, 0.f, 2, c.s);
}

// K5: M <- (M+G) - (1-mu) A B^T and X <- X - eta sqrt(m/n) A B2^T in one pass (A: m x r, B and B2: n x r).
// Large-tile path: bf16 operands from the *16 slots; otherwise fp32 operands from the *32 slots.
// sketch: instead of the weight update, X (which then is a scratch buffer) receives A B^T itself.
int stage_k5(const RowCtx& c, int a16, int b16, int b2_16, int a32, int b32, int b2_32, float mu, float eta,
             bool sketch = false) {
  const Group& g = *c.g;
  const int m = (int)g.m, n = (int)g.n, r = (int)g.r;
  GemmArgs a = c.base;
  a.M = m; a.N = n; a.K = r;
  a.E.slotX = SLOT_X; a.E.slotG = SLOT_G; a.E.slotM = SLOT_M; a.E.ld = n;
  a.E.c_m = 1.0f - mu;
  a.E.c_x = (float)((double)eta * sqrt((double)g.m / (double)g.n));
  if (sketch) {
    a.E.c_x = -1.f;
    a.E.x_overwrite = 1;
    b2_16 = b16;
    b2_32 = b32;
  }
  a.status_slot = SLOT_STATUS;
  if (c.big) {
    a.A = opnd(a16, 0, r);
    a.B = opnd(b16, 0, r);
    a.B2 = opnd(b2_16, 0, r);
    a.xcd_remap = 1;
    // M, X and G of this call beyond what the 256 MB last-level cache can hold from one step to the next: stream them
    a.E.stream_hint = (double)c.batch * (double)m * (double)n * 18.0 > 192e6 ? 1 : 0;
    // Tiles are visited column group by column group, all row tiles of a group before the next group: the n x r column
    // panels of a group (128 rows x r, two bf16 matrices per tile column) are shared by the tiles that run at the same
    // time on an XCD and stay in its L2 from one row of tiles to the next.  About 2.5 MB of panels per group, and at
    // least three tile columns: measured at r = 768 (6 wide), 1024 (5), 2048 and 4096 (3), each against narrower and
    // wider groups and against the plain row-major order, which costs 10 % at r >= 2048.
    a.group_n = (int)(2621440LL / (128LL * r * 4));
    if (a.group_n < 3) a.group_n = 3;
    // (128x128 tiles, two workgroups per compute unit so that one multiplies while the other streams M, G and X, cost
    // twice the operand traffic of the 256x128 tile and lose or tie at every shape measured: 2 % at 8192 x 8192 r = 512,
    // 10 % at r = 768 and 1024, 20 % at r = 2048, even at 2048 x 2048 r = 512)
    HIPCHK(gemm2_k5(G2_256x256, c.gbf16, a, c.batch, c.s));
  } else {
    a.A = opnd(a32, 0, r);
    a.B = opnd(b32, 0, r);
    a.B2 = opnd(b2_32, 0, r);
    HIPCHK(gemm_k5(pick_variant(m, n, r, c.batch, true), c.bf16, c.gbf16, a, c.batch, c.s));
  }
  return DION_OK;
}

#define STAGECHK(expr)            \
  do {                            \
    int rc_ = (expr);             \
    if (rc_ != DION_OK) return rc_; \
  } while (0)

// One Dion step (Algorithm 1 with the unsharded update rule) for the matrices of one shape group.
// The two stages of a Double Dion step (Section 5.2) are such steps with a twist each:
//   STEP_SKETCH     the X buffer is a scratch matrix that receives P R^T instead of a weight update (stage 1)
//   STEP_KEEP_STATUS the status words hold the outcome of stage 1; the orthonormalisation tolerates linearly dependent
//                    columns, since this stage's buffer is a sum of a few low-rank sketches at first (stage 2)
// The status words are cleared by the kernel that refreshes the pointer table before the step.
enum { STEP_PLAIN = 0, STEP_SKETCH = 1, STEP_KEEP_STATUS = 2 };
int step_rows(dion_state* st, int gi, int row0, int batch, float mu, float eta, hipStream_t s, int mode = STEP_PLAIN) {
  const RowCtx c = make_ctx(st, gi, row0, batch, s);
  const Group& g = *c.g;
  const int m = (int)g.m, n = (int)g.n, r = (int)g.r;
  if (c.ev) st->group_timed[gi] = 1;
  STAGECHK(mark(c, DION_STAGE_K1_BQ, 0));
  const int parts = k1_parts_mode(c);
  if (!parts) STAGECHK(stage_b16(c));
  const float rank_tol = mode == STEP_KEEP_STATUS ? RANK_TOL : 0.f;
  bool z_split = false;
  STAGECHK(stage_k1(c, true, SLOT_Q, orth_fuses(c, g.m, g.gram_m, rank_tol), &z_split, parts));
  STAGECHK(mark(c, DION_STAGE_K1_BQ, 1));
  STAGECHK(mark(c, DION_STAGE_ORTH, 0));
  STAGECHK(stage_orth(c, g.m, g.gram_m, SLOT_Z, SLOT_P1, SLOT_P, rank_tol, z_split));
  // bf16 copies of P for K2 and K5.  When the last Cholesky-QR pass found its input orthonormal enough, that input is
  // P, and the pass has left the very same copies (the high parts of its split) in the same two slots.
  // (The product with (M + G)^T on the direct-load path reads the row-major copy; the 128-wide-tile kernel needs the
  // transposed one, which the split leaves only when the Gram matrix took that kernel too.)
  if (c.big) {
    const bool d12 = direct12(c);
    const bool split_left_pt16 = !choose_gram(g, batch, g.m, g.gram_m).big;
    HIPCHK(launch_convert_bf16(c.tab, NSLOTS, batch, SLOT_P, SLOT_P16, d12 ? -1 : SLOT_PT16, m, r, s,
                               (d12 || split_left_pt16) ? SLOT_FAST : -1));
  }
  STAGECHK(mark(c, DION_STAGE_ORTH, 1));
  STAGECHK(mark(c, DION_STAGE_K2_BTP, 0));
  int colsq_chunks = 0;
  STAGECHK(stage_k2(c, SLOT_P, true, &colsq_chunks));
  STAGECHK(mark(c, DION_STAGE_K2_BTP, 1));
  STAGECHK(mark(c, DION_STAGE_COLNORM, 0));
  if (colsq_chunks > 0) HIPCHK(launch_colnorm_final(c.tab, NSLOTS, batch, colsq_chunks, r, s));   // K2 has left the partial sums
  else HIPCHK(launch_colnorm(c.tab, NSLOTS, batch, SLOT_R, n, r, s));
  // (dependent columns: P and R have zero columns there, which add nothing to the update; Q keeps its old column)
  HIPCHK(launch_scale_cols(c.tab, NSLOTS, batch, SLOT_R, SLOT_Q, n, r, SLOT_STATUS, c.big ? SLOT_Q16 : -1, c.big ? SLOT_R16 : -1, s,
                           rank_tol > 0.f ? SLOT_NULL : -1));
  STAGECHK(mark(c, DION_STAGE_COLNORM, 1));
  STAGECHK(mark(c, DION_STAGE_K5_UPDATE, 0));
  STAGECHK(stage_k5(c, SLOT_P16, SLOT_R16, SLOT_Q16, SLOT_P, SLOT_R, SLOT_Q, mu, eta, mode == STEP_SKETCH));
  STAGECHK(mark(c, DION_STAGE_K5_UPDATE, 1));
  return DION_OK;
}

// One Lazy-Dion step (Section 5.1) for the matrices of one shape group; the caller's Q buffer holds V.
//   refresh:  V <- Orthonormalize(B^T (B V))                 (SymPowerIter1; K1, K2 and the orthonormalisation on n x r)
//   always:   W = B V;  M <- B - (1-mu) W V^T;  X <- X - eta sqrt(m/n) ColNorm(W) V^T
// ColNorm(W) V^T = W (V diag(d))^T with d_j = 1 / (||W_j|| + eps), so the fused update kernel of the Dion step
// serves unchanged with A = W, B = V, B2 = V diag(d).
int lazy_rows(dion_state* st, int gi, int row0, int batch, float mu, float eta, bool refresh, hipStream_t s) {
  const RowCtx c = make_ctx(st, gi, row0, batch, s);
  const Group& g = *c.g;
  const int m = (int)g.m, n = (int)g.n, r = (int)g.r;
  if (c.ev) st->group_timed[gi] = 1;
  // the refresh is reported as the orthonormalisation stage; there is no separate K2 stage in this variant
  STAGECHK(mark(c, DION_STAGE_ORTH, 0));
  // (the bf16 copy of M + G either here, or in parts beside the first product that reads it)
  const int parts = k1_parts_mode(c);
  if (!parts) STAGECHK(stage_b16(c));
  if (refresh) {
    STAGECHK(stage_k1(c, true, SLOT_Q, false, nullptr, parts));                   // Z = B V
    if (c.big) HIPCHK(launch_convert_bf16(c.tab, NSLOTS, batch, SLOT_Z, direct12(c) ? SLOT_P16 : -1, direct12(c) ? -1 : SLOT_PT16, m, r, s));
    STAGECHK(stage_k2(c, SLOT_Z));                                                // R = B^T Z
    const int fin = (st->orth_mode == DION_ORTH_SHIFTED_CHOLQR3) ? SLOT_P1 : SLOT_R;
    STAGECHK(stage_orth(c, g.n, g.gram_n, SLOT_R, SLOT_P1, fin));
    // V is state: it only changes when the factorisation succeeded
    HIPCHK(launch_copy_gated(c.tab, NSLOTS, batch, fin, SLOT_Q, (long long)n * r, SLOT_STATUS, s));
  }
  STAGECHK(mark(c, DION_STAGE_ORTH, 1));
  STAGECHK(mark(c, DION_STAGE_K2_BTP, 0));
  STAGECHK(mark(c, DION_STAGE_K2_BTP, 1));
  STAGECHK(mark(c, DION_STAGE_K1_BQ, 0));
  STAGECHK(stage_k1(c, false, SLOT_Q, false, nullptr, refresh ? K1_WHOLE : parts));        // W = B V
  STAGECHK(mark(c, DION_STAGE_K1_BQ, 1));
  STAGECHK(mark(c, DION_STAGE_COLNORM, 0));
  HIPCHK(launch_colnorm(c.tab, NSLOTS, batch, SLOT_Z, m, r, s));                  // d from the columns of W
  // R <- V diag(d) (fp32), with bf16 copies of it and of V for the large-tile update kernel
  HIPCHK(launch_scale_cols(c.tab, NSLOTS, batch, SLOT_Q, SLOT_R, n, r, SLOT_STATUS, c.big ? SLOT_Q16 : -1, c.big ? SLOT_R16 : -1, s));
  if (c.big) HIPCHK(launch_convert_bf16(c.tab, NSLOTS, batch, SLOT_Z, SLOT_P16, -1, m, r, s));
  STAGECHK(mark(c, DION_STAGE_COLNORM, 1));
  STAGECHK(mark(c, DION_STAGE_K5_UPDATE, 0));
  STAGECHK(stage_k5(c, SLOT_P16, SLOT_R16, SLOT_Q16, SLOT_Z, SLOT_Q, SLOT_R, mu, eta));
  STAGECHK(mark(c, DION_STAGE_K5_UPDATE, 1));
  return DION_OK;
}

// One Dion step in the transposed form (Section 4.3, other variants) for the matrices of one shape group; the
// caller's factor buffer holds Vt (m x r):
//   Z' = B^T Vt (n x r);  P' = orth(Z');  R' = B P' (m x r);  M <- B - (1-mu) R' P'^T;  Vt <- ColNorm(R');
//   X <- X - eta sqrt(m/n) Vt_new P'^T = X - eta sqrt(m/n) R' (P' diag(d))^T
// i.e. the products of the standard step in the other order, the orthonormalisation on n x r, and the fused
// update kernel with A = R', B = P', B2 = P' diag(d).
int transposed_rows(dion_state* st, int gi, int row0, int batch, float mu, float eta, hipStream_t s) {
  const RowCtx c = make_ctx(st, gi, row0, batch, s);
  const Group& g = *c.g;
  const int m = (int)g.m, n = (int)g.n, r = (int)g.r;
  if (c.ev) st->group_timed[gi] = 1;
  // stage names as in the standard step: "K2" is the product with B^T, "K1" the one with B
  STAGECHK(mark(c, DION_STAGE_K2_BTP, 0));
  STAGECHK(stage_b16(c));
  if (c.big) HIPCHK(launch_convert_bf16(c.tab, NSLOTS, batch, SLOT_Q, direct12(c) ? SLOT_P16 : -1, direct12(c) ? -1 : SLOT_PT16, m, r, s));
  STAGECHK(stage_k2(c, SLOT_Q, false));                                           // R = B^T Vt   (n x r)
  STAGECHK(mark(c, DION_STAGE_K2_BTP, 1));
  STAGECHK(mark(c, DION_STAGE_ORTH, 0));
  const int pt = (st->orth_mode == DION_ORTH_SHIFTED_CHOLQR3) ? SLOT_P1 : SLOT_R;   // where P' ends up
  const int scratch = (pt == SLOT_R) ? SLOT_P1 : SLOT_R;                            // the other n x r buffer
  STAGECHK(stage_orth(c, g.n, g.gram_n, SLOT_R, SLOT_P1, pt));
  STAGECHK(mark(c, DION_STAGE_ORTH, 1));
  STAGECHK(mark(c, DION_STAGE_K1_BQ, 0));
  STAGECHK(stage_k1(c, false, pt));                                               // Z = B P'     (m x r)
  STAGECHK(mark(c, DION_STAGE_K1_BQ, 1));
  STAGECHK(mark(c, DION_STAGE_COLNORM, 0));
  HIPCHK(launch_colnorm(c.tab, NSLOTS, batch, SLOT_Z, m, r, s));
  // scratch <- P' diag(d) with bf16 copies of it and of P'; Vt <- R' diag(d) with a bf16 copy of R'
  HIPCHK(launch_scale_cols(c.tab, NSLOTS, batch, pt, scratch, n, r, SLOT_STATUS, c.big ? SLOT_Q16 : -1, c.big ? SLOT_R16 : -1, s));
  HIPCHK(launch_scale_cols(c.tab, NSLOTS, batch, SLOT_Z, SLOT_Q, m, r, SLOT_STATUS, -1, c.big ? SLOT_P16 : -1, s));
  STAGECHK(mark(c, DION_STAGE_COLNORM, 1));
  STAGECHK(mark(c, DION_STAGE_K5_UPDATE, 0));
  STAGECHK(stage_k5(c, SLOT_P16, SLOT_R16, SLOT_Q16, SLOT_Z, pt, scratch, mu, eta));
  STAGECHK(mark(c, DION_STAGE_K5_UPDATE, 1));
  return DION_OK;
}

int any_step_rows(dion_state* st, int gi, int row0, int batch, float mu, float eta, hipStream_t s) {
  return st->groups[gi].form == DION_FORM_TRANSPOSED ? transposed_rows(st, gi, row0, batch, mu, eta, s)
                                                     : step_rows(st, gi, row0, batch, mu, eta, s);
}

bool aligned16(const void* p) { return p && ((uintptr_t)p & 15u) == 0; }
bool coeffs_ok(float mu, float eta) { return mu >= 0.f && mu <= 1.f && isfinite(eta) && isfinite(mu); }

bool batch_args_ok(const dion_state* st, int count, void* const* X, const void* const* G, void* const* M, void* const* Q,
                   const int64_t* m, const int64_t* n, const int64_t* r, float mu, float eta) {
  if (count != st->count || !X || !G || !M || !Q || !m || !n || !r || !coeffs_ok(mu, eta)) return false;
  for (int i = 0; i < count; ++i) {
    const Entry& e = st->entries[i];
    if (m[i] != e.m || n[i] != e.n || r[i] != e.r) return false;
    if (!aligned16(X[i]) || !aligned16(G[i]) || !aligned16(M[i]) || !aligned16(Q[i])) return false;
  }
  return true;
}

}  // namespace

extern "C" {

int dion_workspace_bytes(int count, const int64_t* m, const int64_t* n, const int64_t* r, int g_dtype, int math,
                         size_t* bytes_out) {
  if (!bytes_out || !shapes_ok(count, m, n, r)) return DION_EINVAL;
  if ((g_dtype != DION_G_F32 && g_dtype != DION_G_BF16) || (math != DION_MATH_F32 && math != DION_MATH_BF16)) return DION_EINVAL;
  try {
    std::vector<Entry> entries;
    std::vector<Group> groups;
    build_plan(count, m, n, r, nullptr, math, entries, groups);   // the form does not change any size
    size_t total = header_bytes(count);
    for (auto& g : groups) total += g.bytes_per_entry * g.count;
    *bytes_out = total + 256;
  } catch (const std::bad_alloc&) {
    return DION_ENOMEM;
  }
  return DION_OK;
}

int dion_init_state(dion_state_t** out, int count, const int64_t* m, const int64_t* n, const int64_t* r, int g_dtype,
                    int math, void* workspace_dev, size_t workspace_bytes, void* const* M_dev, void* const* Q_dev,
                    int q_is_filled, uint64_t seed, void* hip_stream) {
  return dion_init_state_ex(out, count, m, n, r, nullptr, g_dtype, math, workspace_dev, workspace_bytes, M_dev, Q_dev,
                            q_is_filled, seed, hip_stream);
}

int dion_init_state_ex(dion_state_t** out, int count, const int64_t* m, const int64_t* n, const int64_t* r, const int* form,
                       int g_dtype, int math, void* workspace_dev, size_t workspace_bytes, void* const* M_dev,
                       void* const* Q_dev, int q_is_filled, uint64_t seed, void* hip_stream) {
  if (!out) return DION_EINVAL;
  if (form)
    for (int i = 0; i < count; ++i)
      if (form[i] != DION_FORM_STANDARD && form[i] != DION_FORM_TRANSPOSED) return DION_EINVAL;
  *out = nullptr;
  size_t need = 0;
  int rc = dion_workspace_bytes(count, m, n, r, g_dtype, math, &need);
  if (rc != DION_OK) return rc;
  if (count > 0 && (!M_dev || !Q_dev)) return DION_EINVAL;
  if (!workspace_dev || ((uintptr_t)workspace_dev & 255u)) return DION_EINVAL;
  if (workspace_bytes < need) return DION_EWORKSPACE;
  for (int i = 0; i < count; ++i)
    if (!aligned16(M_dev[i]) || !aligned16(Q_dev[i])) return DION_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  // kernels that use more than 64 KB of LDS are given leave to do so now, not at their first launch, which may
  // be inside a stream capture
  if (gemm2_nt_prepare() != hipSuccess || gemm2_k5_prepare() != hipSuccess) return DION_ELAUNCH;
  dion_state* st = nullptr;
  try {
    st = new dion_state();
    std::vector<void*> host;
    const int prc = plan_state(st, count, m, n, r, form, g_dtype, math, workspace_dev, workspace_bytes, M_dev, Q_dev, host);
    if (prc != DION_OK) {
      delete st;
      return prc;
    }
    st->last_stream = s;
    const unsigned long long zero = 0;
    if (hipMemcpy(st->step_counter, &zero, sizeof(zero), hipMemcpyHostToDevice) != hipSuccess ||
        (count > 0 && hipMemcpy(st->table, host.data(), host.size() * sizeof(void*), hipMemcpyHostToDevice) != hipSuccess)) {
      delete st;
      return DION_ELAUNCH;
    }
  } catch (const std::bad_alloc&) {
    delete st;
    return DION_ENOMEM;
  }
  for (const Group& g : st->groups)
    if (g.direct12) {
      create_side_stream(st);
      break;
    }
  // device-side initialisation: M = 0, Q = ColNorm(Q or Gaussian draw)
  auto fail = [&](int code) { destroy_side_stream(st); delete st; return code; };
  for (int i = 0; i < count; ++i) {
    const Entry& e = st->entries[i];
    void* const* rowtab = st->table + (size_t)e.row * NSLOTS;
    if (launch_fill(rowtab, NSLOTS, 1, SLOT_M, (long long)e.m * e.n, 0.f, s) != hipSuccess) return fail(DION_ELAUNCH);
    if (!q_is_filled)
      if (launch_gaussian_fill(rowtab, NSLOTS, 1, SLOT_Q, (e.form == DION_FORM_TRANSPOSED ? e.m : e.n) * e.r, seed, i, s) != hipSuccess) return fail(DION_ELAUNCH);
  }
  for (auto& g : st->groups) {
    void* const* tab = st->table + (size_t)g.first_row * NSLOTS;
    if (launch_fill_i32(tab, NSLOTS, g.count, SLOT_STATUS, 1, 0, s) != hipSuccess) return fail(DION_ELAUNCH);
    if (launch_fill(tab, NSLOTS, g.count, SLOT_SYNC, 2 * sync_words(g.rp / CHOL_NB), 0.f, s) != hipSuccess) return fail(DION_ELAUNCH);
    if (launch_fill(tab, NSLOTS, g.count, SLOT_W, (long long)g.rp * g.rp, 0.f, s) != hipSuccess) return fail(DION_ELAUNCH);
    const long long frows = g.form == DION_FORM_TRANSPOSED ? g.m : g.n;   // the factor is n x r, or m x r in the transposed form
    if (launch_colnorm(tab, NSLOTS, g.count, SLOT_Q, frows, (int)g.r, s) != hipSuccess) return fail(DION_ELAUNCH);
    if (launch_scale_cols(tab, NSLOTS, g.count, SLOT_Q, SLOT_Q, frows, (int)g.r, -1, -1, -1, s) != hipSuccess) return fail(DION_ELAUNCH);
  }
  *out = st;
  return DION_OK;
}

int dion_step_batched(dion_state_t* st, int count, void* const* X, const void* const* G, void* const* M, void* const* Q,
                      const int64_t* m, const int64_t* n, const int64_t* r, float mu, float eta, void* hip_stream) {
  if (!st || count < 0) return DION_EINVAL;
  if (count == 0) return DION_OK;
  if (!batch_args_ok(st, count, X, G, M, Q, m, n, r, mu, eta)) return DION_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  st->last_stream = s;
  std::fill(st->group_timed.begin(), st->group_timed.end(), 0);
  try {
    // user pointers in table-row order
    std::vector<void*> xs(count), ms(count), qs(count);
    std::vector<const void*> gs(count);
    for (int i = 0; i < count; ++i) {
      const int row = st->entries[i].row;
      xs[row] = X[i]; gs[row] = G[i]; ms[row] = M[i]; qs[row] = Q[i];
    }
    HIPCHK(launch_set_user_ptrs(st->table, NSLOTS, 0, count, xs.data(), gs.data(), ms.data(), qs.data(), s, st->status, st->step_counter));
  } catch (const std::bad_alloc&) {
    return DION_ENOMEM;
  }
  for (size_t gi = 0; gi < st->groups.size(); ++gi) {
    int rc = any_step_rows(st, (int)gi, 0, st->groups[gi].count, mu, eta, s);
    if (rc != DION_OK) return rc;
  }
  return DION_OK;
}

int dion_step(dion_state_t* st, void* X, const void* G, void* M, void* Q, int64_t m, int64_t n, int64_t r, float mu,
              float eta, void* hip_stream) {
  if (!st || !coeffs_ok(mu, eta)) return DION_EINVAL;
  if (!aligned16(X) || !aligned16(G) || !aligned16(M) || !aligned16(Q)) return DION_EINVAL;
  int idx = -1;
  for (int i = 0; i < st->count && idx < 0; ++i)
    if (st->entries[i].m == m && st->entries[i].n == n && st->entries[i].r == r) idx = i;
  if (idx < 0) return DION_EINVAL;
  const Entry& e = st->entries[idx];
  const Group& g = st->groups[e.group];
  hipStream_t s = (hipStream_t)hip_stream;
  st->last_stream = s;
  std::fill(st->group_timed.begin(), st->group_timed.end(), 0);
  void* xs[1] = {X};
  const void* gs[1] = {G};
  void* ms[1] = {M};
  void* qs[1] = {Q};
  HIPCHK(launch_set_user_ptrs(st->table, NSLOTS, e.row, 1, xs, gs, ms, qs, s, st->status, st->step_counter));
  return any_step_rows(st, e.group, e.row - g.first_row, 1, mu, eta, s);
}

int dion_lazy_step_batched(dion_state_t* st, int count, void* const* X, const void* const* G, void* const* M, void* const* V,
                           const int64_t* m, const int64_t* n, const int64_t* r, float mu, float eta, int refresh,
                           void* hip_stream) {
  if (!st || count < 0) return DION_EINVAL;
  if (count == 0) return DION_OK;
  if (!batch_args_ok(st, count, X, G, M, V, m, n, r, mu, eta)) return DION_EINVAL;
  for (const Group& g : st->groups)
    if (g.form != DION_FORM_STANDARD) return DION_EINVAL;   // Lazy-Dion is built for the standard form only
  hipStream_t s = (hipStream_t)hip_stream;
  st->last_stream = s;
  std::fill(st->group_timed.begin(), st->group_timed.end(), 0);
  try {
    std::vector<void*> xs(count), ms(count), qs(count);
    std::vector<const void*> gs(count);
    for (int i = 0; i < count; ++i) {
      const int row = st->entries[i].row;
      xs[row] = X[i]; gs[row] = G[i]; ms[row] = M[i]; qs[row] = V[i];
    }
    HIPCHK(launch_set_user_ptrs(st->table, NSLOTS, 0, count, xs.data(), gs.data(), ms.data(), qs.data(), s, st->status, st->step_counter));
  } catch (const std::bad_alloc&) {
    return DION_ENOMEM;
  }
  for (size_t gi = 0; gi < st->groups.size(); ++gi) {
    int rc = lazy_rows(st, (int)gi, 0, st->groups[gi].count, mu, eta, refresh != 0, s);
    if (rc != DION_OK) return rc;
  }
  return DION_OK;
}

int dion_lazy_step(dion_state_t* st, void* X, const void* G, void* M, void* V, int64_t m, int64_t n, int64_t r, float mu,
                   float eta, int refresh, void* hip_stream) {
  if (!st || !coeffs_ok(mu, eta)) return DION_EINVAL;
  if (!aligned16(X) || !aligned16(G) || !aligned16(M) || !aligned16(V)) return DION_EINVAL;
  int idx = -1;
  for (int i = 0; i < st->count && idx < 0; ++i)
    if (st->entries[i].m == m && st->entries[i].n == n && st->entries[i].r == r) idx = i;
  if (idx < 0 || st->entries[idx].form != DION_FORM_STANDARD) return DION_EINVAL;
  const Entry& e = st->entries[idx];
  const Group& g = st->groups[e.group];
  hipStream_t s = (hipStream_t)hip_stream;
  st->last_stream = s;
  std::fill(st->group_timed.begin(), st->group_timed.end(), 0);
  void* xs[1] = {X};
  const void* gs[1] = {G};
  void* ms[1] = {M};
  void* qs[1] = {V};
  HIPCHK(launch_set_user_ptrs(st->table, NSLOTS, e.row, 1, xs, gs, ms, qs, s, st->status, st->step_counter));
  return lazy_rows(st, e.group, e.row - g.first_row, 1, mu, eta, refresh != 0, s);
}

int dion_double_step(dion_state_t* st1, dion_state_t* st2, int count, void* const* X, const void* const* G, void* const* M1,
                     void* const* V1, void* const* M2, void* const* V2, void* const* D, const int64_t* m, const int64_t* n,
                     const int64_t* r1, const int64_t* r2, float mu1, float mu2, float eta, void* hip_stream) {
  if (!st1 || !st2 || count < 0) return DION_EINVAL;
  if (count == 0) return DION_OK;
  if (!D || st2->g_dtype != DION_G_F32) return DION_EINVAL;   // the sketch is an fp32 matrix
  if (!batch_args_ok(st1, count, D, G, M1, V1, m, n, r1, mu1, eta)) return DION_EINVAL;
  if (!batch_args_ok(st2, count, X, (const void* const*)D, M2, V2, m, n, r2, mu2, eta)) return DION_EINVAL;
  for (const Group& g : st1->groups) if (g.form != DION_FORM_STANDARD) return DION_EINVAL;
  for (const Group& g : st2->groups) if (g.form != DION_FORM_STANDARD) return DION_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  st1->last_stream = st2->last_stream = s;
  std::fill(st1->group_timed.begin(), st1->group_timed.end(), 0);
  std::fill(st2->group_timed.begin(), st2->group_timed.end(), 0);
  try {
    std::vector<void*> xs(count), ms(count), qs(count);
    std::vector<const void*> gs(count);
    std::vector<int> rows1(count), rows2(count);
    // stage 1: a Dion step of rank r1 on (M1, V1) whose "weights" are the sketch buffer D
    for (int i = 0; i < count; ++i) {
      const int row = st1->entries[i].row;
      xs[row] = D[i]; gs[row] = G[i]; ms[row] = M1[i]; qs[row] = V1[i];
      rows1[i] = row;
      rows2[i] = st2->entries[i].row;
    }
    HIPCHK(launch_set_user_ptrs(st1->table, NSLOTS, 0, count, xs.data(), gs.data(), ms.data(), qs.data(), s, st1->status, st1->step_counter));
    for (size_t gi = 0; gi < st1->groups.size(); ++gi) {
      int rc = step_rows(st1, (int)gi, 0, st1->groups[gi].count, mu1, 0.f, s, STEP_SKETCH);
      if (rc != DION_OK) return rc;
    }
    // stage 2: a Dion step of rank r2 on (X, M2, V2) with D as its gradient, skipped where stage 1 failed
    HIPCHK(launch_copy_status_rows(st1->status, st2->status, count, rows1.data(), rows2.data(), s));
    for (int i = 0; i < count; ++i) {
      const int row = st2->entries[i].row;
      xs[row] = X[i]; gs[row] = D[i]; ms[row] = M2[i]; qs[row] = V2[i];
    }
    HIPCHK(launch_set_user_ptrs(st2->table, NSLOTS, 0, count, xs.data(), gs.data(), ms.data(), qs.data(), s, nullptr, st2->step_counter));
    for (size_t gi = 0; gi < st2->groups.size(); ++gi) {
      int rc = step_rows(st2, (int)gi, 0, st2->groups[gi].count, mu2, eta, s, STEP_KEEP_STATUS);
      if (rc != DION_OK) return rc;
    }
  } catch (const std::bad_alloc&) {
    return DION_ENOMEM;
  }
  return DION_OK;
}

int dion_retry_breakdowns(dion_state_t* st, int count, void* const* X, const void* const* G, void* const* M,
                          void* const* Q, const int64_t* m, const int64_t* n, const int64_t* r, float mu, float eta,
                          void* hip_stream, int* retried_out) {
  if (!st || count < 0) return DION_EINVAL;
  if (retried_out) *retried_out = 0;
  if (count == 0) return DION_OK;
  if (!batch_args_ok(st, count, X, G, M, Q, m, n, r, mu, eta)) return DION_EINVAL;
  HIPCHK(hipStreamSynchronize(st->last_stream));
  hipStream_t s = (hipStream_t)hip_stream;
  std::vector<int> host;
  try {
    host.resize(count);
  } catch (const std::bad_alloc&) {
    return DION_ENOMEM;
  }
  HIPCHK(hipMemcpy(host.data(), st->status, sizeof(int) * count, hipMemcpyDeviceToHost));
  st->last_stream = s;
  std::fill(st->group_timed.begin(), st->group_timed.end(), 0);
  const int saved_mode = st->orth_mode;
  int retried = 0, rc = DION_OK;
  for (int i = 0; i < count && rc == DION_OK; ++i) {
    const Entry& e = st->entries[i];
    if (host[e.row] == 0) continue;
    const Group& g = st->groups[e.group];
    // a wait that timed out says nothing about the matrix: same orthonormalisation, without the kernels that wait;
    // a breakdown: the shifted three-pass variant
    st->force_panel = host[e.row] == ST_TIMEOUT;
    st->orth_mode = st->force_panel ? saved_mode : DION_ORTH_SHIFTED_CHOLQR3;
    void* xs[1] = {X[i]};
    const void* gs[1] = {G[i]};
    void* ms[1] = {M[i]};
    void* qs[1] = {Q[i]};
    if (launch_set_user_ptrs(st->table, NSLOTS, e.row, 1, xs, gs, ms, qs, s, st->status, st->step_counter) != hipSuccess) { rc = DION_ELAUNCH; break; }
    rc = any_step_rows(st, e.group, e.row - g.first_row, 1, mu, eta, s);
    ++retried;
  }
  st->orth_mode = saved_mode;
  st->force_panel = false;
  if (retried_out) *retried_out = retried;
  return rc;
}

int dion_last_status(dion_state_t* st, int* status_out, int* first_bad_index) {
  if (!st) return DION_EINVAL;
  HIPCHK(hipStreamSynchronize(st->last_stream));
  int status = DION_OK, bad = -1;
  if (st->count > 0) {
    try {
      std::vector<int> host(st->count);
      HIPCHK(hipMemcpy(host.data(), st->status, sizeof(int) * st->count, hipMemcpyDeviceToHost));
      for (int i = 0; i < st->count && bad < 0; ++i)
        if (host[st->entries[i].row] != 0) {
          status = host[st->entries[i].row] == ST_TIMEOUT ? DION_WAIT_TIMEOUT : DION_NUM_BREAKDOWN;
          bad = i;
        }
    } catch (const std::bad_alloc&) {
      return DION_ENOMEM;
    }
  }
  if (status_out) *status_out = status;
  if (first_bad_index) *first_bad_index = bad;
  return DION_OK;
}

int dion_set_orth_mode(dion_state_t* st, int mode) {
  if (!st || (mode != DION_ORTH_CHOLQR2 && mode != DION_ORTH_SHIFTED_CHOLQR3 && mode != DION_ORTH_CHOLQR2_FALLBACK)) return DION_EINVAL;
  st->orth_mode = mode;
  return DION_OK;
}

int dion_cholesky_grid(int compute_units, int batch, int64_t r, int* workgroups_out) {
  if (compute_units < 1 || batch < 1 || r < 1 || r > 32768 || !workgroups_out) return DION_EINVAL;
  int pr = 0, pc = 0, chain = 0;
  plan_chol_grid(compute_units, batch, padded_rank(r) / CHOL_NB, &pr, &pc, &chain);
  *workgroups_out = pr * pc + chain;
  return DION_OK;
}

int dion_set_wait_limit(dion_state_t* st, unsigned polls) {
  if (!st) return DION_EINVAL;
  st->chol_spin_limit = polls;
  return DION_OK;
}

int dion_measure_ceilings(void* scratch_dev, size_t scratch_bytes, double* mfma_tflops, double* stream_gbps, void* hip_stream) {
  if (!scratch_dev || ((uintptr_t)scratch_dev & 255u) || !mfma_tflops || !stream_gbps) return DION_EINVAL;
  if (scratch_bytes < (size_t)10 * (1u << 20)) return DION_EWORKSPACE;
  const long long elems = (long long)(scratch_bytes / 10);
  if (run_ceiling_probes(scratch_dev, elems, mfma_tflops, stream_gbps, (hipStream_t)hip_stream) != hipSuccess) return DION_ELAUNCH;
  return DION_OK;
}

int dion_set_stage_timing(dion_state_t* st, int enable) {
  if (!st) return DION_EINVAL;
  if (enable && st->events.empty()) {
    try {
      st->events.resize(st->groups.size() * kEventsPerGroup, nullptr);
    } catch (const std::bad_alloc&) {
      return DION_ENOMEM;
    }
    for (auto& e : st->events) HIPCHK(hipEventCreate(&e));
  }
  st->timing = enable != 0;
  return DION_OK;
}

int dion_stage_times(dion_state_t* st, float* ms_out) {
  if (!st || !ms_out) return DION_EINVAL;
  for (int i = 0; i < DION_STAGE_COUNT; ++i) ms_out[i] = 0.f;
  if (st->events.empty()) return DION_EINVAL;
  HIPCHK(hipStreamSynchronize(st->last_stream));
  for (size_t gi = 0; gi < st->groups.size(); ++gi) {
    if (!st->group_timed[gi]) continue;
    hipEvent_t* ev = &st->events[gi * kEventsPerGroup];
    for (int sidx = 0; sidx < DION_STAGE_COUNT; ++sidx) {
      float ms = 0.f;
      HIPCHK(hipEventElapsedTime(&ms, ev[2 * sidx], ev[2 * sidx + 1]));
      ms_out[sidx] += ms;
    }
  }
  return DION_OK;
}

int dion_debug_buffer(dion_state_t* st, int index, int which, void** ptr_out, int64_t* ld_out) {
  if (!st || index < 0 || index >= st->count || !ptr_out) return DION_EINVAL;
  static const int slots[] = {SLOT_Z, SLOT_P, SLOT_R, SLOT_S, SLOT_STATUS, SLOT_P1, SLOT_C, SLOT_L, SLOT_W, SLOT_D, SLOT_NULL};
  if (which < 0 || which >= (int)(sizeof(slots) / sizeof(slots[0]))) return DION_EINVAL;
  const Entry& e = st->entries[index];
  void* p = nullptr;
  HIPCHK(hipMemcpy(&p, st->table + (size_t)e.row * NSLOTS + slots[which], sizeof(void*), hipMemcpyDeviceToHost));
  *ptr_out = p;
  if (ld_out) {
    const int sl = slots[which];
    *ld_out = (sl == SLOT_C || sl == SLOT_L || sl == SLOT_W) ? st->groups[e.group].rp
              : (sl == SLOT_S || sl == SLOT_D || sl == SLOT_STATUS || sl == SLOT_NULL) ? 1 : e.r;
  }
  return DION_OK;
}

int dion_destroy_state(dion_state_t* st) {
  if (!st) return DION_OK;
  for (auto& e : st->events)
    if (e) (void)hipEventDestroy(e);
  destroy_side_stream(st);
  delete st;
  return DION_OK;
}

const char* dion_strerror(int code) {
  switch (code) {
    case DION_OK: return "ok";
    case DION_EINVAL: return "invalid argument";
    case DION_EWORKSPACE: return "workspace too small";
    case DION_ELAUNCH: return "HIP runtime error";
    case DION_ENOMEM: return "host allocation failed";
    case DION_NUM_BREAKDOWN: return "Cholesky breakdown: Z rank deficient or too ill conditioned";
    case DION_WAIT_TIMEOUT: return "a wait between workgroups timed out: the GPU could not keep a single-launch kernel resident";
    default: return "unknown code";
  }
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------------------
// dion_step_static: the Dion step on a workspace that lives in the library itself.
constexpr size_t kStaticScratchBytes = DION_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
// What the library knows about the static workspace of one device.  `ptr` is the array's address on that device
// (hipGetSymbolAddress; the array's name itself means nothing in host code); `st` is the host-side plan of the shape
// the last call used, carved over `ptr`.
struct StaticSlot {
  bool ready;
  unsigned char* ptr;
  dion_state* st;
  int64_t m, n, r;
  int g_dtype, math;
};
StaticSlot g_static[16];
}  // namespace

extern "C" int dion_step_static(void* X, const void* G, void* M, void* Q, int64_t m, int64_t n, int64_t r, int g_dtype, int math,
                                float mu, float eta, int* status_dev, void* hip_stream) {
  if (!coeffs_ok(mu, eta)) return DION_EINVAL;
  if (!aligned16(X) || !aligned16(G) || !aligned16(M) || !aligned16(Q)) return DION_EINVAL;
  if (status_dev && ((uintptr_t)status_dev & 3u)) return DION_EINVAL;
  size_t need = 0;
  int rc = dion_workspace_bytes(1, &m, &n, &r, g_dtype, math, &need);   // validates the shape and the two type codes
  if (rc != DION_OK) return rc;
  if (need > kStaticScratchBytes) return DION_EWORKSPACE;              // beyond what the static workspace holds
  int dev = 0;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= 16) return DION_EINVAL;
  StaticSlot& slot = g_static[dev];
  hipStream_t s = (hipStream_t)hip_stream;
  if (!slot.ready) {
    // set-up, once per device, with that device current: every GPU has its own copy of the array at its own address
    void* p = nullptr;
    HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255u)) return DION_ELAUNCH;
    if (gemm2_nt_prepare() != hipSuccess || gemm2_k5_prepare() != hipSuccess) return DION_ELAUNCH;
    slot.ptr = (unsigned char*)p;
    slot.st = nullptr;
    slot.ready = true;
  }
  if (!slot.st || slot.m != m || slot.n != n || slot.r != r || slot.g_dtype != g_dtype || slot.math != math) {
    // another shape than last time: a new host-side plan over the same memory (host memory only)
    dion_state* st = nullptr;
    try {
      st = new dion_state();
      std::vector<void*> host;
      rc = plan_state(st, 1, &m, &n, &r, nullptr, g_dtype, math, slot.ptr, kStaticScratchBytes, nullptr, nullptr, host);
      if (rc == DION_OK && launch_set_table_row(st->table, host.data(), s) != hipSuccess) rc = DION_ELAUNCH;
    } catch (const std::bad_alloc&) {
      rc = DION_ENOMEM;
    }
    if (rc != DION_OK) {
      delete st;
      return rc;
    }
    delete slot.st;
    slot.st = st;
    slot.m = m; slot.n = n; slot.r = r; slot.g_dtype = g_dtype; slot.math = math;
  }
  dion_state* st = slot.st;
  st->last_stream = s;
  const Group& g = st->groups[0];
  // The array keeps what the last call left there, of whatever shape: everything that a step expects to find zero is
  // cleared by fill kernels (no memset: the call may be captured).  The step counter, at a fixed place at the start of
  // the array, is never cleared: it only has to differ from one call to the next.
  HIPCHK(launch_fill(st->table, NSLOTS, 1, SLOT_SYNC, 2 * sync_words(g.rp / CHOL_NB), 0.f, s));
  HIPCHK(launch_fill(st->table, NSLOTS, 1, SLOT_W, (long long)g.rp * g.rp, 0.f, s));
  void* xs[1] = {X};
  const void* gs[1] = {G};
  void* ms[1] = {M};
  void* qs[1] = {Q};
  HIPCHK(launch_set_user_ptrs(st->table, NSLOTS, 0, 1, xs, gs, ms, qs, s, st->status, st->step_counter));
  rc = step_rows(st, 0, 0, 1, mu, eta, s);
  if (rc != DION_OK) return rc;
  if (status_dev) HIPCHK(launch_copy_i32(st->status, status_dev, s));
  return DION_OK;
}
