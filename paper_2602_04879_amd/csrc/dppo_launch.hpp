// Host-side launch entry points of the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "dppo_common.hpp"

namespace dppo {

// General two-pass kernel.  vec=false selects the element-wise variant (needed when logits
// and grad_logits rows do not share their 16-byte misalignment).
hipError_t launch_streaming(const KParams& p, bool vec, bool grad, int threads, int grid, hipStream_t s);

// Register-resident kernel (fused forward+backward, or forward only).  A shape is (threads per workgroup, 16-byte
// chunks per thread); resident_shape() picks the smallest instantiated one that covers a row of
// V entries (false: none does).  ragged = false: V a multiple of 8 and 16-byte aligned rows of logits and
// grad.  ragged = true: any V, any pitch, rows 2-byte aligned; logits and grad must share their
// misalignment (address mod 16); the kernel reads the aligned 128-byte lines that hold a row and
// writes the row's own entries only.  resident_blocks_per_cu() is the occupancy the runtime reports
// for a shape (dyn: of the form that hands its rows out at run time).
bool resident_shape(int64_t V, bool ragged, int* threads, int* chunks);
hipError_t launch_resident(const KParams& p, bool grad, bool ragged, int threads, int chunks, int grid, hipStream_t s);
int resident_blocks_per_cu(bool grad, bool dyn, bool ragged, int threads, int chunks);

// Register-resident kernel for rows too long for the register file alone (forward+backward only):
// part of the row in registers, part in LDS, the rest passed through twice.  resident_long_chunks()
// gives the number of 512 x 16-byte chunks of a row this form takes, 0 where it does not apply
// (V not a multiple of 8, or outside 155 657 .. 262 144).  Needs 16-byte aligned rows of logits and
// grad; one workgroup per compute unit.
int resident_long_chunks(int64_t V);
hipError_t launch_resident_long(const KParams& p, int chunks, int grid, hipStream_t s);

// Register-resident kernel for rows of middle length (forward+backward only): groups of `rows`
// consecutive rows of `chunks` x 512 x 16 bytes each per workgroup, one workgroup per compute unit,
// groups handed out at run time, one loss term per row (p.row_counters and p.row_loss must be set).  resident_multi_shape()
// gives the group shape for a row of V entries, false where the form does not apply (V not a
// multiple of 8, or not within two chunks of 1024 entries below 24576, 32768, 40960, 49152, 57344 or 65536).  Needs 16-byte aligned rows of logits and grad.
// ragged: as for the one-row kernel.
bool resident_multi_shape(int64_t V, bool ragged, int* rows, int* chunks);
hipError_t launch_resident_multi(const KParams& p, bool ragged, int rows, int chunks, int grid, hipStream_t s);

// Two-row kernel of the exact full-vocabulary variants (tv: total variation, else KL).
hipError_t launch_fullvocab(const KParams& p, bool tv, bool grad, int threads, int grid, hipStream_t s);

// Register-resident form of the same variants (backward, and the forward-only TV form): the
// trainer's row in the registers of one workgroup of 512 threads per compute unit, the rollout row
// streamed past it.  fullvocab_resident_chunks() says whether a call qualifies (0: no) and with
// how many 16-byte chunks per thread.
int fullvocab_resident_chunks(const KParams& p, bool tv, bool grad);
hipError_t launch_fullvocab_resident(const KParams& p, bool tv, bool grad, int chunks, int grid, hipStream_t s);

// bf16 matrix products on the matrix cores (fp32 accumulation).  A, B 16-byte aligned with lda, ldb
// multiples of 8 and 256 * ld * 2 < 2^32; the fp32 forms need 16-byte aligned rows of C.
// C[M, N] = A B^T, A [M, K], B [N, K]; K % 64 == 0; out 0: C bf16; 1: C fp32; 2: C fp32, added to what it holds
hipError_t launch_gemm_nt(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, int out, hipStream_t s);
// C[M, N] bf16 = A B, A [M, K], B [K, N]; K % 64 == 0
hipError_t launch_gemm_nn(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, hipStream_t s);
// C[M, N] fp32 (out 1: written, 2: added to) = A^T B, A [K, M], B [K, N]; any K >= 1
hipError_t launch_gemm_tn(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, int out, hipStream_t s);

// Clears the eight row counters of the register-resident kernel's run-time row hand-out.
hipError_t launch_clear_counters(int32_t* counters, hipStream_t s);

// What the first product of the hidden-state path leaves instead of logits (forward only): per row
// and 256-column tile the statistics (b, s, t, -) of the bf16-rounded logits of that tile, the
// sampled token's own term left out (b: integer offset -ceil(max * log2e); s = sum 2^(z*log2e + b);
// t = sum 2^x * x), and the rounded logits at the row's sampled id and top-K ids.
typedef float gemm_f32x4 __attribute__((ext_vector_type(4)));
struct GemmStats {
  gemm_f32x4* part = nullptr;        // [M][tiles_n]
  float* gath = nullptr;             // [M][Ktop + 1]: column 0 the sampled id, 1..Ktop the top-K ids; ids outside [0, N) leave their entry unwritten
  const int32_t* sampled = nullptr;  // [M]
  const int32_t* tk_ids = nullptr;   // [M][Ktop] (unused if Ktop = 0)
  int32_t Ktop = 0, tiles_n = 0;
};
constexpr int kGemmTileN = 256;
hipError_t launch_gemm_stats(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, int M, int N, int K,
                             const GemmStats& gs, hipStream_t s);
// Per row: combine the tiles' statistics and run the per-row epilogue (one wave per row).  p holds the
// per-token arrays of the rows (logits unused), row_loss [p.T] receives the loss terms.
hipError_t launch_lmhead_rows(const KParams& p, const GemmStats& gs, double* row_loss, hipStream_t s);

// loss[0] = loss_scale * sum(partial[0..n)) in a fixed order.
hipError_t launch_finalize(const double* partial, int n, float loss_scale, float* loss, hipStream_t s);

}  // namespace dppo
