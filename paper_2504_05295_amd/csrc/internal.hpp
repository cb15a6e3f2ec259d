// Declarations shared by the translation units of libdion.so (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_core.hpp"

namespace dion {

// Pointer-table slots of one matrix parameter.  Slots 0-3 are the caller's buffers and are
// refreshed on every step; the rest point into the workspace and are fixed at init.
enum Slot {
  SLOT_X = 0, SLOT_G, SLOT_M, SLOT_Q,
  SLOT_Z,      // Z = B Q                      m x r
  SLOT_P1,     // Z after the first Cholesky-QR pass
  SLOT_P,      // P = orth(Z)                  m x r
  SLOT_R,      // R = B^T P                    n x r
  SLOT_C,      // Gram matrix                  rp x rp  (rp = padded r)
  SLOT_L,      // its Cholesky factor          rp x rp
  SLOT_W,      // L^-1                         rp x rp
  SLOT_T,      // scratch of the inverse       rp x rp
  SLOT_CPART,  // split-K partial Gram matrices
  SLOT_SPART,  // partial column sums of squares
  SLOT_S,      // column norms of R            r
  SLOT_D,      // 1 / (s + eps)                r
  SLOT_STATUS, // int32 breakdown flag
  SLOT_QT16,   // Q^T as bf16                  r x n   (B operand of K1, k = n contiguous)
  SLOT_P16,    // P as bf16                    m x r   (A operand of K5)
  SLOT_PT16,   // P^T as bf16                  r x m   (B operand of K2, k = m contiguous)
  SLOT_R16,    // R as bf16                    n x r   (B operand of K5)
  SLOT_Q16,    // Q_new as bf16                n x r   (second B operand of K5)
  // split-bf16 copies used by the orthonormalisation in bf16 mode (x = hi + lo, both bf16).  The hi parts
  // of the m x r matrix live in SLOT_P16 / SLOT_PT16, which are free until P is final.
  SLOT_ZL16,   // lo part                      m x r
  SLOT_ZLT16,  // lo part, transposed          r x m
  SLOT_WH16,   // hi part of L^-1              r x r
  SLOT_WL16,   // lo part of L^-1              r x r
  SLOT_EPART,  // GRAM_DEFECT_PARTS partial sums of the squared Gram defect ||C - I||_F^2
  SLOT_FAST,   // int32: 1 when the last Cholesky-QR pass found its input orthonormal to the tolerance
  SLOT_KPART,  // split-K partial results of K1 / K2 (small outputs that cannot fill the GPU otherwise)
  SLOT_SYNC,   // flags of the single-launch Cholesky factorisation (64-bit words)
  SLOT_B16,    // bf16(M + G), m x n: operand of K1 and (read with k as the slow index) of K2 on the direct-load path; else
               // written by K1 on its way for K2
  SLOT_THR,    // rp floats: pivot thresholds of the factorisation that tolerates dependent columns
  SLOT_NULL,   // rp int32: 1 for the columns that factorisation found dependent on the ones before them
  SLOT_GATE,   // int32: 0 when the orthonormalisation of this matrix has to be redone by the fallback passes, else 1
  NSLOTS = 40
};

// Values of a matrix' device status word (SLOT_STATUS).  0 = fine; anything else gates the state-writing kernels.
enum StatusWord {
  ST_OK = 0,
  ST_BREAKDOWN = 1,   // a Cholesky pivot outside its bounds: numerical property of the matrix
  ST_TIMEOUT = 2,     // a bounded wait inside a single-launch kernel gave up: scheduling, not numerics
  ST_UPSTREAM = 3     // Double Dion: the first stage of this matrix failed, the second was not attempted
};

constexpr int CHOL_NB = 64;        // Cholesky panel width (diagonal block factored by one wavefront)
constexpr float COLNORM_EPS = 1e-8f;
constexpr float RANK_TOL = 1e-3f;   // a pivot at most this fraction of the Gram matrix' own diagonal entry: dependent column
constexpr int GRAM_DEFECT_PARTS = 1024;   // workgroups (and partial sums) of the kernel that measures ||C - I||_F
constexpr int COLNORM_ROWS = 256;  // rows per partial sum of squares (colnorm_partial_kernel)
constexpr int COLNORM_CHUNK_MIN = 128;   // fewest rows per partial sum that any producer uses (sizes SLOT_SPART)

// Tile configurations of the MFMA GEMM core.
using CfgBig = TileCfg<128, 128, 32, 2, 2>;
using CfgSmall = TileCfg<64, 64, 64, 2, 2>;
enum { VAR_BIG = 0, VAR_SMALL = 1, VAR_SMALL_CHECKED = 2 };

// Picks the tile variant for a product with output M x N and contraction K whose operands all
// have leading dimensions that are multiples of 8 whenever the dimensions are multiples of 64.
int pick_variant(long long M, long long N, long long K, long long batch, bool aligned);

// GEMM families (each defined in its own translation unit).  `bf16`: MMA operand type.
hipError_t gemm_k1(int variant, bool bf16, bool gbf16, GemmArgs g, int batch, hipStream_t s);   // A = M+G (KC), B = fp32 KS
hipError_t gemm_k2(int variant, bool bf16, bool gbf16, GemmArgs g, int batch, hipStream_t s);   // A = M+G (KS), B = fp32 KS
hipError_t gemm_k5(int variant, bool bf16, bool gbf16, GemmArgs g, int batch, hipStream_t s);   // dual B, fused update
// Large-tile bf16 versions (gemm_core2.hpp); `cfg` selects the tile, see gemm2_*.hip.  They return
// hipErrorInvalidValue when the shape is not a multiple of the tile.
enum { G2_256x256 = 0, G2_128x128 = 1, G2_256x128 = 2 };   // (the last one: gemm2_nt only)
hipError_t gemm2_k1(int cfg, bool gbf16, GemmArgs g, int batch, hipStream_t s);
hipError_t gemm2_k2(int cfg, bool gbf16, GemmArgs g, int batch, hipStream_t s, bool from_bf16 = false);   // from_bf16: A = bf16 [K][M]
hipError_t gemm2_k5(int cfg, bool gbf16, GemmArgs g, int batch, hipStream_t s);
int gemm2_k1_splitk(int cfg, const GemmArgs& g);   // number of split-K partials the launch will write
int gemm2_k2_splitk(int cfg, const GemmArgs& g);
// measured ceilings: bf16 MFMA issue loop (TFLOP/s) and an 18-byte-per-element streaming pass (GB/s); synchronises
hipError_t run_ceiling_probes(void* scratch, long long elems, double* mfma_tflops, double* stream_gbps, hipStream_t s);
// dynamic-LDS permissions of the direct-load kernels on the current device (once per device; not inside a capture)
hipError_t gemm2_nt_prepare();
hipError_t gemm2_k5_prepare();
// bf16 A x bf16 B, up to 3 operand pairs; element (row, k) of an operand at p[row * ld + k], or, for the operands named
// in `ks` (KS_A | KS_B; 256 x 256 tiles of the direct-load core only), at p[k * ld + row]
enum { KS_A = 1, KS_B = 2 };
hipError_t gemm2_nt(int cfg, GemmArgs g, int batch, hipStream_t s, int ks = 0);
// rows of per-column partial sums of squares that gemm2_nt writes for these arguments when GemmArgs::E.colsq_slot is set
// (0: this product cannot, leave the slot at -1)
int gemm2_nt_colsq_chunks(int cfg, const GemmArgs& g, int ks = 0);
// true when gemm2_nt (ks = 0) will run these arguments on the direct-load core, whose plain-store epilogue can also leave
// the result split into bf16 halves (EpilogueDesc::split_hi1 / split_lo1)
bool gemm2_nt_is_direct(int cfg, const GemmArgs& g);
int gemm2_nt_splitk(int cfg, const GemmArgs& g);                       // number of split-K partials gemm2_nt will write
hipError_t gemm_f32_nt(int variant, GemmArgs g, int batch, hipStream_t s);                      // A KC, B KC
hipError_t gemm_f32_nn(int variant, GemmArgs g, int batch, hipStream_t s);                      // A KC, B KS
hipError_t gemm_f32_tn(int variant, GemmArgs g, int batch, hipStream_t s);                      // A KS, B KS

// Small kernels (small_kernels.hip).  All take the pointer table and a batch count.
// status != nullptr: clears status[first_row .. first_row + count) as well; counter != nullptr: increments that word
hipError_t launch_set_user_ptrs(void** table, int nslots, int first_row, int count, void* const* X, const void* const* G,
                                void* const* M, void* const* Q, hipStream_t s, int* status, unsigned long long* counter);
// table[0 .. NSLOTS) = values[0 .. NSLOTS) (host array), by a kernel whose arguments carry the values
hipError_t launch_set_table_row(void** table, void* const* values, hipStream_t s);
hipError_t launch_copy_i32(const int* src, int* dst, hipStream_t s);   // *dst = *src on the device
// count_slot >= 0: also adds one to the 64-bit word number count_index of that slot (a launch counter kept on the device)
// dst_status[dst_rows[i]] = 2 where src_status[src_rows[i]] != 0, else 0, for i < count (row lists are host arrays)
hipError_t launch_copy_status_rows(const int* src_status, int* dst_status, int count, const int* src_rows, const int* dst_rows,
                                   hipStream_t s);
// SLOT_THR[j] = tol * C[j][j] for j < rp (C = SLOT_C, before it is factored)
hipError_t launch_rank_threshold(void* const* table, int nslots, int batch, int rp, float tol, hipStream_t s);
// Per matrix: a status word that reports a numerical breakdown is cleared and SLOT_GATE set to 0 (the fallback passes that
// follow redo this matrix; SLOT_FAST is cleared too, so that the copies made of their result are not skipped); every
// other matrix gets SLOT_GATE = 1.
hipError_t launch_fallback_decide(void* const* table, int nslots, int batch, hipStream_t s);
hipError_t launch_fill(void* const* table, int nslots, int batch, int slot, long long count, float value, hipStream_t s);
// out <- in unless *status != 0 (both 16-byte aligned)
hipError_t launch_copy_gated(void* const* table, int nslots, int batch, int slot_in, int slot_out, long long count, int status_slot,
                             hipStream_t s);
// out16 = bf16(M + G) as [rows][cols]  (rows * cols a multiple of 8)
hipError_t launch_sum_bf16(void* const* table, int nslots, int batch, int slot_m, int slot_g, bool gbf16, int slot_out16,
                           long long rows, long long cols, hipStream_t s);
// ... for the columns [col_first, col_first + col_count) (multiples of 8) of the rows [row_first, row_first + row_count) only
hipError_t launch_sum_bf16_cols(void* const* table, int nslots, int batch, int slot_m, int slot_g, bool gbf16, int slot_out16,
                                long long rows, long long cols, long long row_first, long long row_count, long long col_first,
                                long long col_count, hipStream_t s);
hipError_t launch_fill_i32(void* const* table, int nslots, int batch, int slot, long long count, int value, hipStream_t s);
// C[j][j] += shift_rel * trace(C[0:r,0:r]) for j < r (shifted Cholesky-QR); the trace is summed in a fixed order
// (skip_slot >= 0 here and below: the int32 there non-zero means that the launch leaves this matrix alone)
hipError_t launch_shift_diagonal(void* const* table, int nslots, int batch, int r, int rp, float shift_rel, hipStream_t s, int skip_slot = -1);
hipError_t launch_pad_identity(void* const* table, int nslots, int batch, int slot, int r, int rp, hipStream_t s, int skip_slot = -1);
hipError_t launch_reduce_partials(void* const* table, int nslots, int batch, int slot_part, int slot_out, int r, long long ld,
                                  int nsplit, long long split_stride, hipStream_t s, int skip_slot = -1);
// out = sum over `nsplit` partial matrices of `count` floats each, stored back to back in slot_part (fixed order)
hipError_t launch_sum_partials(void* const* table, int nslots, int batch, int slot_part, int slot_out, long long count,
                               int nsplit, hipStream_t s);
hipError_t launch_colnorm(void* const* table, int nslots, int batch, int slot_in, long long rows, int r, hipStream_t s);
// second stage alone: s, d from nchunks rows of partial sums of squares already in SLOT_SPART
hipError_t launch_colnorm_final(void* const* table, int nslots, int batch, int nchunks, int r, hipStream_t s);
// out = in diag(d) (fp32), optional bf16 copies of out and of in.  null_slot >= 0: columns whose int32 there is
// non-zero keep their old fp32 values in `out` (the bf16 copies still receive in diag(d))
hipError_t launch_scale_cols(void* const* table, int nslots, int batch, int slot_in, int slot_out, long long rows, int r,
                             int status_slot, int slot_out16, int slot_in16, hipStream_t s, int null_slot = -1);
// fp32 [rows][cols] -> bf16 copy [rows][cols] (slot_out16 >= 0) and bf16 transpose [cols][rows] (slot_outT16 >= 0);
// rows and cols must be multiples of 64.
// fp32 [rows][cols] (leading dimension ld_in) -> split bf16 x = hi + lo: plain copies [rows][cols] and transposed
// copies [cols][rows]; any output slot may be -1.  rows and cols must be multiples of 64.
hipError_t launch_split_bf16(void* const* table, int nslots, int batch, int slot_in, long long ld_in, long long rows,
                             long long cols, int slot_hi, int slot_lo, int slot_hiT, int slot_loT, hipStream_t s,
                             int skip_slot = -1);   // skip_slot >= 0: nothing happens for matrices whose int32 there is non-zero
hipError_t launch_convert_bf16(void* const* table, int nslots, int batch, int slot_in, int slot_out16, int slot_outT16,
                               long long rows, long long cols, hipStream_t s, int skip_slot = -1);
hipError_t launch_gaussian_fill(void* const* table, int nslots, int batch, int slot, long long count, uint64_t seed,
                                int first_stream, hipStream_t s);
// Buffers of the first matrix of a batch; matrix b has them `stride` 4-byte words further (status: b ints further).
// skip != nullptr: the launch does nothing for matrices whose int32 there is non-zero.
struct CholPanelPtrs {
  float* C;
  float* L;
  float* W;
  int* status;
  const int* skip;
  long long stride;
  // both null: a pivot outside its bounds is a breakdown.  Else (rp entries per matrix, `stride` words apart): a pivot
  // not above thr[j] marks column j as dependent on the columns before it; it is left out of the factorisation (zero
  // column of L, zero row and column of the inverse) and nullmask[j] is set, otherwise cleared.
  const float* thr;
  int* nullmask;
};
hipError_t launch_chol_panel(CholPanelPtrs p, int batch, int k0, int rp, float piv_lo, float piv_hi, hipStream_t s);
// The whole factorisation in one launch (tiles owned by pr x pc workgroups that hand results on through flags).
// sync: per matrix chol_sync_words(rp / 64) 64-bit words that were zero before the first launch: flags and the abort word.
// Flags are tagged with *step_counter * 8 + pass: the counter is a device word that a kernel increments once per
// step (on the device, so that a captured graph can be replayed), pass (1..7) tells the launches of one step
// apart.  Every wait inside the kernel gives up after spin_limit polls.
// All pr * pc * batch workgroups must fit on the GPU at once.
struct CholStreamArgs {
  float* C;
  float* L;
  float* W;
  int* status;
  const int* skip;
  unsigned long long* sync;
  long long stride;        // 4-byte words between the matrices of a batch (C, L, W, skip)
  long long sync_stride;   // 64-bit words between their flag arrays
  int rp, pr, pc;
  float piv_lo, piv_hi;
  const unsigned long long* step_counter;
  int pass;
  unsigned spin_limit;
  const float* thr;        // as in CholPanelPtrs
  int* nullmask;
  int chain;               // 1: one more workgroup, number 0, carries the whole chain of diagonal blocks (pr x pc helpers)
  int vflag_off;           // chain only: > 0: the helpers form W = L^-1 as well (no inverse pass afterwards), and (rp / 64)^2
                           // flag words for it start this many 64-bit words into the matrix' sync array; 0: they do not
#ifdef DION_CHOL_TIMING
  long long* dbg;          // timing build only: eight time stamps per panel of the chain workgroup
#endif
};
hipError_t launch_chol_stream(CholStreamArgs p, int batch, hipStream_t s);
// W = L^-1 from L and the inverses of its 64 x 64 diagonal blocks (both as the factorisation leaves them), one launch
// for `batch` matrices with `groups` workgroups each; groups * batch must not exceed the number of compute units.
constexpr int INV_TREE_MAX_GROUPS = 256;
struct InvTreeArgs {
  const float* L;
  float* W;
  float* T;                // scratch, rp x rp
  int* status;
  const int* skip;         // per matrix: non-zero = nothing to do (or nullptr)
  unsigned long long* sync;   // per matrix INV_TREE_MAX_GROUPS arrival words + 1 abort word
  long long stride;        // 4-byte words between the matrices of a batch (L, W, T, skip)
  long long sync_stride;   // 64-bit words between their arrival words
  int rp;
  const unsigned long long* step_counter;
  int pass;
  unsigned spin_limit;
};
hipError_t launch_inv_tree(InvTreeArgs p, int groups, int batch, int cus, hipStream_t s);
// Workgroup grid pr x pc per matrix of the single-launch factorisation (and pr * pc groups for the inverse) for `batch`
// matrices of nb 64-wide panels on a GPU with `cus` compute units; pr = 0: use a launch per panel instead.  All
// pr * pc * batch workgroups must be resident at once, one per compute unit.
// *chain = 1: pr x pc helper workgroups plus one that carries the chain of diagonal blocks (pr * pc + 1 in all).
void plan_chol_grid(int cus, int batch, int nb, int* pr, int* pc, int* chain);
// 64-bit words of SLOT_SYNC for a matrix with nb 64-wide panels: the factorisation's flags, then the inverse's
constexpr int chol_sync_words(int nb) { return 3 * nb + 2; }
constexpr int FUSED_INV_MAX_NB = 64;   // most panels for which the factorisation kernel forms the inverse as well (< 256:
                                       // its waits take one thread per panel)
constexpr int fused_inv_flag_offset(int nb) { return chol_sync_words(nb) + INV_TREE_MAX_GROUPS + 2; }
constexpr int sync_words(int nb) { return fused_inv_flag_offset(nb) + (nb <= FUSED_INV_MAX_NB ? nb * nb : 0); }
// Second Cholesky-QR pass shortcut.  When the Gram matrix C of the first pass' output is within tau of the identity in
// Frobenius norm, SLOT_FAST is set to 1 (else 0) and, unless decision_only, W receives chol(C)^-1 = I - Phi(C - I) up to
// O(tau^2), Phi = strict lower part + half the diagonal.  nsplit > 1: C still is nsplit split-K partial results in
// SLOT_CPART, split_stride words apart; their sum is formed (and stored to SLOT_C) here.
hipError_t launch_first_order_inverse(void* const* table, int nslots, int batch, int r, int rp, float tau, bool decision_only,
                                      int nsplit, long long split_stride, hipStream_t s);

}  // namespace dion
