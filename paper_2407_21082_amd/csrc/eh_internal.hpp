// Host-side internals shared by the translation units of libeh.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "eh.h"
#include "eh_device.hpp"

struct CalibScratch {
  void* buf = nullptr;
  size_t bytes = 0;
  int* host_flag = nullptr;   // pinned: the refinement's "tables too small" word
  long long n_sorted = 0;     // calls that the full sort served
};

struct eh_ctx {
  int d = 0, V = 0, n_heads = 0, max_rows = 0, dtype = 0, device = 0;
  float eps = 1e-5f;
  int KS = 0, VT = 0, R_pad_max = 0;
  int num_cu = 0;
  bool use_gemm = true;
  std::vector<eh::frag_t*> Wf;  // per head, fragment-major weights
  std::vector<float*> gamma, beta, bias;
  std::vector<float> tau;
  // device-side copies of the per-head tables (read by the persistent kernel)
  eh::frag_t** d_Wf = nullptr;
  float** d_gamma = nullptr;
  float** d_beta = nullptr;
  float** d_bias = nullptr;
  float* d_tau = nullptr;
  eh::frag_t* yf = nullptr;     // [R_pad_max/16][KS][64] activations in fragment order
  eh::Stats* partials = nullptr;  // [kStreamGrid][R_pad_max]
  // workspace of eh_eval_heads, allocated by its first call: one activation buffer and one
  // set of partials per head
  eh::frag_t* mh_yf = nullptr;
  eh::Stats* mh_partials = nullptr;
  float* mh_second = nullptr;  // second largest logits, same shape as mh_partials
  int mh_heads = 0;
  CalibScratch calib;  // eh_calibrate's scratch, grown on demand
  // workspace of eh_head_losses, allocated by its first call: partial statistics
  // [kStreamGrid][R_pad_max] and the per-token loss terms [2][R_pad_max]
  eh::KlStats* kl_partials = nullptr;
  float* kl_rows = nullptr;
  float* ws_H = nullptr;        // [max_rows] internal outputs (cascade, verify)
  float* ws_lse = nullptr;
  int* ws_argmax = nullptr;
  int* active[2] = {nullptr, nullptr};
  int* n_active[2] = {nullptr, nullptr};
  // persistent decode kernel: control block and per-head partials
  int decode_grid = 0;          // 0 = shape not supported by the decode kernel
  size_t decode_smem = 0;
  unsigned long long* dec_records = nullptr;  // [2 rounds][n_heads][decode_grid][16][5] {tag, payload} words
  int* dec_status = nullptr;                // sticky device-side failure flag
  unsigned dec_epoch = 0;
  int spin_limit = 1 << 22;                 // polls of another workgroup's record before giving up
  unsigned long long* dec_trace = nullptr;  // [n_heads][16] timestamps of workgroup 0 (diagnostics)
  int dec_trace_on = 0;
  // persistent kernel for 17 .. 256 rows (bf16, no bias): 0 = shape not supported
  int rows_grid = 0;
  int* rows_ctl = nullptr;             // control block (counters, live-row masks), cleared before each launch
  int* rows_vctl = nullptr;            // two control blocks of a verification, used in turn: a launch clears the other one
  int rows_vctl_ints = 0;              // size of one of them
  unsigned rows_vturn = 0;             // verifications launched so far
  int rows_ctl_ints = 0;
  eh::frag_t* rows_y = nullptr;        // [n_heads][rows_y_stride] activations, one buffer per head
  long long rows_y_stride = 0;         // fragments
  eh::frag_t* rows_part4 = nullptr;    // [2][rows_grid][256] partial statistics of two consecutive heads: (m, S, U, zb)
  int* rows_parti = nullptr;           // [2][rows_grid][256]: ib
  void* static_scratch = nullptr;  // device address of the library's static workspace on this device
  std::vector<void*> allocs;
  std::string err = "";
};

namespace eh {

// Arguments of the persistent decode kernel (<= 16 rows, heads l0 .. l1-1).
struct DecodeParams {
  const frag_t* const* Wf;
  const float* const* gamma;
  const float* const* beta;
  const float* const* bias;  // nullable
  const float* tau;
  const void* h;
  long long layer_stride, row_stride;  // elements
  const int* row_idx;                  // nullable gather list (evaluation mode)
  const int* n_rows_dev;               // nullable live-row count
  int n_rows, l0, l1, n_heads, decide;
  int V, d, KS, VT;
  float eps;
  unsigned long long* records;  // [2 rounds][n_heads_alloc][grid][16][5]
  int n_heads_alloc;            // head stride of the record array
  unsigned epoch;               // this launch's tag, never 0
  int* status;
  int spin_limit;               // polls before a wait on another workgroup gives up
  float* H;
  float* lse;
  int* argmax;       // evaluation mode outputs [n_rows]
  int* exit_layer;
  int* token;        // cascade outputs [n_rows]
  float* H_out;      // nullable [n_heads][n_rows]
  unsigned long long* n_evals;  // nullable
  unsigned long long* trace;    // nullable: [n_heads][16] wall-clock stamps written by workgroup 0
};

// Arguments of the persistent kernel for 17 .. 256 rows (bf16 heads without a bias vector):
// heads l0 .. l1-1 of a cascade (mode 0) or the model's head of a verification (mode 1).
constexpr int kRowsMax = 256;
struct RowsParams {
  const frag_t* const* Wf;
  const float* const* gamma;
  const float* const* beta;
  const float* tau;             // device [n_heads]
  const void* h;                // mode 0: [head][row][d] through the strides; mode 1: [rows][d]
  long long layer_stride, row_stride;  // elements
  int n_rows, n_heads, l0, l1, mode, argmax_only;
  int V, d, KS, VT16;
  float eps;
  int n_stream;                 // workgroups that stream weights; the rest of the grid serves
  int spin_limit;
  int* ctl;                     // control block, all zero at launch
  const int* live;              // NULL, or a device word: the launch does nothing if it reads 0 (a draft that has stopped)
  int* ctl_next;                // verification: the block of the next launch, cleared by this one (else NULL)
  int n_ctl_next;
  frag_t* y;                    // [l1 - l0][y_stride]: one buffer per head of the launch
  long long y_stride;
  frag_t* part4;                // [2][n_stream][R_pad]: (m, S, U, zb) of the partial statistics of two consecutive heads
  int* parti;                   // [2][n_stream][R_pad]: their ib
  int R_pad;
  int* status;
  int* exit_layer;              // mode 0 outputs
  int* token;
  float* H_out;                 // nullable [n_heads][n_rows]
  unsigned long long* n_evals;  // nullable
  const int* draft;             // mode 1: [B][k]
  const int* draft_len;         // nullable [B]
  int B, k;
  int* accepted;
  int* next_token;
  int* target;                  // nullable [B][k+1]
};
// Occupancy check and sizes for the rows kernel; leaves ctx->rows_grid = 0 if it cannot run.
hipError_t rows_prepare(eh_ctx* ctx);
// Enqueues the preset of outputs and control block, then the kernel.
hipError_t rows_launch(const eh_ctx* ctx, const RowsParams& p, hipStream_t s);
int rows_control_ints(int n_heads);   // size of the control block for a launch over n_heads heads
int rows_service_workgroups(int n_rows);  // workgroups of a cascade's grid that do not stream

// Sets up the decode kernel for this context (grid, LDS size, function
// attributes).  Leaves ctx->decode_grid = 0 if the shape does not fit.
hipError_t decode_prepare(eh_ctx* ctx);
// Enqueues the batched projection + statistics kernel (fp32) for one head on the rows
// laid out in yf (fragments of 16 rows); per-workgroup partial statistics go to
// partials[*n_parts][n_rows rounded up to 16].  Heads with a bias vector are not supported.
hipError_t gemm_launch(const eh_ctx* ctx, int head, const int* n_rows_dev, int n_rows, bool argmax_only,
                       const eh::frag_t* yf, eh::Stats* partials, int* n_parts, hipStream_t s);
// Same for bf16 with blocks of 32 rows: yf must hold the rows in the 32 x 16 operand
// order (ln_pack_kernel<DtBf16, 32>), partials are [*n_parts][n_rows rounded up to 32].
// `second`: NULL, or [*n_parts][rows rounded up to 32] floats that receive, per workgroup and
// row, the second largest logit (counting multiplicity) of the workgroup's vocabulary slice.
hipError_t gemm32_launch(const eh_ctx* ctx, int head, const int* n_rows_dev, int n_rows, bool argmax_only,
                         const eh::frag_t* yf, eh::Stats* partials, float* second, int* n_parts,
                         hipStream_t s);
// Several consecutive heads in one launch (independent heads: eh_eval_heads): the activations
// of head l lie l * y_stride fragments behind yf, its partials (and second largest logits)
// l * part_stride records behind partials (second).
hipError_t gemm32_launch_heads(const eh_ctx* ctx, int head, int n_heads, const int* n_rows_dev, int n_rows,
                               bool argmax_only, const eh::frag_t* yf, long long y_stride, eh::Stats* partials,
                               float* second, long long part_stride, int* n_parts, hipStream_t s);
// The fused projections of the training objectives (bf16, no bias vector): an exit head on
// yf_head and the model's head on yf_model (both in the 32 x 16 operand order, same rows),
// labels NULL or device [n_rows]; per-workgroup partial statistics go to
// partials[*n_parts][n_rows rounded up to 32].
hipError_t gemm32_kl_launch(const eh_ctx* ctx, int head, int model_head, int n_rows, const eh::frag_t* yf_head,
                            const eh::frag_t* yf_model, const int* labels, eh::KlStats* partials, int* n_parts,
                            hipStream_t s);
// Threshold calibration of one head (eh_calib.hip): device inputs, host eps, device outputs.
// Asynchronous on s; its scratch memory (about 20 bytes per token) lives in `sc`, grows on
// demand (which synchronises the device) and is freed by the owner of `sc`.
hipError_t calibrate_run(CalibScratch& sc, const float* H, const int* pred, const int* ref, int64_t M,
                         const double* eps, int n_eps, float* tau_out, long long* n_exit_out, hipStream_t s);
// Enqueues the decode kernel.
hipError_t decode_launch(const eh_ctx* ctx, const DecodeParams& p, hipStream_t s);

}  // namespace eh

#ifdef EH_DIAGNOSTICS
// Diagnostics build only (-DEH_DIAGNOSTICS; not part of the library's interface): with
// enable != 0 later decode launches make workgroup 0 record 16 wall-clock stamps (100 MHz
// ticks) per head; host_out (host, nullable, n entries) first receives what was recorded
// so far (synchronises the device).
extern "C" eh_status eh_decode_trace(eh_ctx* ctx, int32_t enable, uint64_t* host_out, int32_t n);
#endif

namespace eh {

}  // namespace eh
