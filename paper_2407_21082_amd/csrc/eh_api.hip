// libeh: C ABI and host-side dispatch (see include/eh.h for the contract).
#include "eh.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "eh_internal.hpp"
#include "eh_kernels.hpp"

using namespace eh;

// Workspace of eh_eval_noalloc: one array per GPU, part of the library's image on that GPU
// from the moment the library is loaded there until the process ends.  Host code never uses
// this name as an address: eh_create looks the array's device address up once per device
// (scratch_address) and everything is done through that pointer.
constexpr size_t kNoAllocScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

namespace {

thread_local std::string g_create_error = "";

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device.
hipError_t scratch_address(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

constexpr int kMaxNB = 10;           // token blocks (of 16) one stream launch covers
constexpr int kStreamGrid = 512;     // workgroups of the stream kernel (2 per CU)

struct DeviceGuard {
  int prev = -1;
  bool changed = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) == hipSuccess && prev != dev) {
      changed = (hipSetDevice(dev) == hipSuccess);
    }
  }
  ~DeviceGuard() {
    if (changed) (void)hipSetDevice(prev);
  }
};

}  // namespace

namespace {

eh_status fail(eh_ctx* ctx, eh_status st, const std::string& msg) {
  if (ctx) ctx->err = msg; else g_create_error = msg;
  return st;
}

#define EH_HIP(ctx, call)                                                             \
  do {                                                                                \
    hipError_t e_ = (call);                                                           \
    if (e_ != hipSuccess)                                                             \
      return fail(ctx, EH_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
  } while (0)

template <typename T>
hipError_t dev_alloc(eh_ctx* ctx, T** p, size_t count) {
  void* v = nullptr;
  hipError_t e = hipMalloc(&v, count * sizeof(T) > 0 ? count * sizeof(T) : 16);
  if (e == hipSuccess) {
    ctx->allocs.push_back(v);
    *p = (T*)v;
  }
  return e;
}

void free_all(eh_ctx* ctx) {
  for (void* p : ctx->allocs) (void)hipFree(p);
  ctx->allocs.clear();
  if (ctx->calib.buf) (void)hipFree(ctx->calib.buf);
  if (ctx->calib.host_flag) (void)hipHostFree(ctx->calib.host_flag);
  ctx->calib = CalibScratch();
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

template <typename DT, bool AO>
void launch_stream(int nbc, const eh_ctx* c, int head, int nb0, const int* n_rows_dev, int n_rows,
                   int R_pad, hipStream_t s, const frag_t* yf, Stats* partials) {
  const frag_t* Wf = c->Wf[head];
  const float* bias = c->bias.empty() ? nullptr : c->bias[head];
  dim3 g(kStreamGrid), b(256);
#define EH_LAUNCH(NB)                                                                           \
  hipLaunchKernelGGL((stream_kernel<DT, NB, AO>), g, b, 0, s, Wf, yf, bias, c->VT, c->KS, c->V, \
                     nb0, n_rows_dev, n_rows, R_pad, partials)
  if (nbc <= 1) EH_LAUNCH(1);
  else if (nbc <= 2) EH_LAUNCH(2);
  else if (nbc <= 4) EH_LAUNCH(4);
  else if (nbc <= 6) EH_LAUNCH(6);
  else if (nbc <= 8) EH_LAUNCH(8);
  else EH_LAUNCH(10);
#undef EH_LAUNCH
}

// LayerNorm + projection + statistics for one head; results to (H, lse, argmax).
// yf / partials: the activation workspace and the per-workgroup partial statistics to use
// (the context's own, or another buffer of at least the same layout for n_rows rows).
template <bool AO>
eh_status run_head(eh_ctx* c, int head, const void* h, int64_t row_stride, const int* row_idx,
                   const int* n_rows_dev, int n_rows, float* H, float* lse, int* argmax,
                   hipStream_t s, frag_t* yf = nullptr, Stats* partials = nullptr) {
  if (!yf) yf = c->yf;
  if (!partials) partials = c->partials;
  const bool bf = c->dtype == EH_BF16;
  // heads without bias go to the batched kernels: bf16 in blocks of 32 rows
  // (32x32x16 matrix instructions), f32 in blocks of 16
  const bool batched = c->bias.empty() && c->use_gemm;
  const int RB = (batched && bf) ? 32 : 16;
  const int R_pad = (n_rows + RB - 1) / RB * RB;
  {
    dim3 g(R_pad), b(kLnThreads);
    if (bf && RB == 32)
      hipLaunchKernelGGL((ln_pack_kernel<DtBf16, 32>), g, b, 0, s, h, row_stride, row_idx, n_rows_dev,
                         n_rows, R_pad, c->d, c->KS, c->gamma[head], c->beta[head], c->eps, yf);
    else if (bf)
      hipLaunchKernelGGL((ln_pack_kernel<DtBf16, 16>), g, b, 0, s, h, row_stride, row_idx, n_rows_dev,
                         n_rows, R_pad, c->d, c->KS, c->gamma[head], c->beta[head], c->eps, yf);
    else
      hipLaunchKernelGGL((ln_pack_kernel<DtF32, 16>), g, b, 0, s, h, row_stride, row_idx, n_rows_dev,
                         n_rows, R_pad, c->d, c->KS, c->gamma[head], c->beta[head], c->eps, yf);
  }
  int n_parts = kStreamGrid;
  if (batched && bf) {
    EH_HIP(c, gemm32_launch(c, head, n_rows_dev, n_rows, AO, yf, partials, nullptr, &n_parts, s));
  } else if (batched) {
    EH_HIP(c, gemm_launch(c, head, n_rows_dev, n_rows, AO, yf, partials, &n_parts, s));
  } else {
    const int NBtot = R_pad / 16;
    for (int nb0 = 0; nb0 < NBtot; nb0 += kMaxNB) {
      const int nbc = std::min(kMaxNB, NBtot - nb0);
      if (bf) launch_stream<DtBf16, AO>(nbc, c, head, nb0, n_rows_dev, n_rows, R_pad, s, yf, partials);
      else launch_stream<DtF32, AO>(nbc, c, head, nb0, n_rows_dev, n_rows, R_pad, s, yf, partials);
    }
  }
  hipLaunchKernelGGL(finalize_kernel, dim3(n_rows), dim3(64), 0, s, partials, n_parts, R_pad,
                     n_rows_dev, n_rows, AO ? nullptr : H, AO ? nullptr : lse, argmax, (int64_t)0, (int64_t)0);
  EH_HIP(c, hipGetLastError());
  return EH_OK;
}

eh_status check_rows(eh_ctx* ctx, const void* h, int64_t row_stride, int n_rows) {
  if (n_rows < 0 || n_rows > ctx->max_rows)
    return fail(ctx, EH_ERR_WORKSPACE, "n_rows outside [0, max_rows]");
  if (row_stride < ctx->d) return fail(ctx, EH_ERR_SHAPE, "row stride smaller than d");
  const int esz = ctx->dtype == EH_BF16 ? 2 : 4;
  if (!aligned16(h) || (row_stride * esz) % 16 != 0)
    return fail(ctx, EH_ERR_SHAPE, "hidden rows must be 16-byte aligned");
  return EH_OK;
}

// Rows <= 16 go through the persistent decode kernel when the shape fits it.
bool use_decode(const eh_ctx* c, int n_rows) { return c->decode_grid > 0 && n_rows <= 16; }
// 17 .. 256 rows of a cascade or a verification go through the persistent rows kernel.
// The persistent kernel for up to 256 rows; at most 16 rows go to the decode kernel where the
// context has one (hidden sizes up to 2048), and here otherwise.
bool use_rows(const eh_ctx* c, int64_t n_rows) {
  return c->rows_grid > 0 && c->use_gemm && (n_rows > 16 || c->decode_grid == 0) && n_rows >= 1 && n_rows <= kRowsMax &&
         n_rows <= c->max_rows;
}

RowsParams rows_base(eh_ctx* c, int n_rows) {
  RowsParams p{};
  p.Wf = c->d_Wf; p.gamma = c->d_gamma; p.beta = c->d_beta; p.tau = c->d_tau;
  p.n_rows = n_rows; p.n_heads = c->n_heads;
  p.V = c->V; p.d = c->d; p.KS = c->KS; p.VT16 = c->VT; p.eps = c->eps;
  p.n_stream = c->rows_grid - rows_service_workgroups(n_rows);
  p.spin_limit = c->spin_limit;
  p.ctl = c->rows_ctl; p.y = c->rows_y; p.y_stride = c->rows_y_stride;
  p.part4 = c->rows_part4; p.parti = c->rows_parti; p.R_pad = (n_rows + 31) & ~31;
  p.status = c->dec_status;
  return p;
}

DecodeParams decode_base(eh_ctx* c) {
  DecodeParams p{};
  p.Wf = c->d_Wf; p.gamma = c->d_gamma; p.beta = c->d_beta; p.bias = c->d_bias; p.tau = c->d_tau;
  p.n_heads = c->n_heads; p.V = c->V; p.d = c->d; p.KS = c->KS; p.VT = c->VT; p.eps = c->eps;
  p.records = c->dec_records; p.n_heads_alloc = c->n_heads;
  if (++c->dec_epoch == 0u) ++c->dec_epoch;  // never 0
  p.epoch = c->dec_epoch; p.status = c->dec_status;
  p.spin_limit = c->spin_limit;
#ifdef EH_DIAGNOSTICS
  p.trace = c->dec_trace_on ? c->dec_trace : nullptr;
#endif
  return p;
}

}  // namespace

extern "C" {

const char* eh_version(void) { return "libeh 0.1 (gfx950)"; }

const char* eh_last_error(const eh_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

eh_status eh_create(const eh_config* cfg, eh_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return fail(nullptr, EH_ERR_NULL, "cfg or out is NULL");
  if (!cfg->W || !cfg->gamma || !cfg->beta || !cfg->tau)
    return fail(nullptr, EH_ERR_NULL, "W, gamma, beta and tau are required");
  if (cfg->d <= 0 || cfg->V <= 0 || cfg->n_heads <= 0 || cfg->max_rows <= 0)
    return fail(nullptr, EH_ERR_SHAPE, "d, V, n_heads and max_rows must be positive");
  if (cfg->w_dtype != EH_F32 && cfg->w_dtype != EH_BF16)
    return fail(nullptr, EH_ERR_DTYPE, "unknown w_dtype");
  if (cfg->w_dtype != cfg->h_dtype)
    return fail(nullptr, EH_ERR_DTYPE, "w_dtype and h_dtype must match");
  const int epl = cfg->w_dtype == EH_BF16 ? 8 : 4;
  const int kpf = 4 * epl;
  if (cfg->d % epl != 0)
    return fail(nullptr, EH_ERR_SHAPE, "d must be a multiple of 16 bytes worth of elements");
  if (!(cfg->ln_eps > 0.f) || !std::isfinite(cfg->ln_eps))
    return fail(nullptr, EH_ERR_RANGE, "ln_eps must be positive and finite");
  if ((int64_t)cfg->max_rows > (1 << 20)) return fail(nullptr, EH_ERR_RANGE, "max_rows too large");
  for (int l = 0; l < cfg->n_heads; ++l) {
    if (!cfg->W[l] || !cfg->gamma[l] || !cfg->beta[l] || (cfg->bias && !cfg->bias[l]))
      return fail(nullptr, EH_ERR_NULL, "a per-head pointer is NULL");
    if (!aligned16(cfg->W[l])) return fail(nullptr, EH_ERR_SHAPE, "W must be 16-byte aligned");
  }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev)
    return fail(nullptr, EH_ERR_RANGE, "no such HIP device");

  eh_ctx* c = new (std::nothrow) eh_ctx();
  if (!c) return fail(nullptr, EH_ERR_HIP, "out of host memory");
  c->d = cfg->d; c->V = cfg->V; c->n_heads = cfg->n_heads; c->max_rows = cfg->max_rows;
  c->dtype = cfg->w_dtype; c->device = cfg->device; c->eps = cfg->ln_eps;
  c->KS = (cfg->d + kpf - 1) / kpf;
  c->VT = (cfg->V + 15) / 16;
  c->R_pad_max = (cfg->max_rows + 31) & ~31;
  c->tau.assign(cfg->tau, cfg->tau + cfg->n_heads);

  DeviceGuard guard(c->device);
  auto bail = [&](hipError_t e, const char* what) {
    std::string msg = std::string(what) + ": " + hipGetErrorString(e);
    free_all(c);
    delete c;
    return fail(nullptr, EH_ERR_HIP, msg);
  };
  hipError_t e;
  if ((e = scratch_address(c->device, &c->static_scratch)) != hipSuccess) return bail(e, "hipGetSymbolAddress(scratch)");
  const size_t wf_frags = (size_t)c->VT * c->KS * kWave;
  const int Vp = c->VT * 16;
  c->Wf.resize(c->n_heads); c->gamma.resize(c->n_heads); c->beta.resize(c->n_heads);
  if (cfg->bias) c->bias.resize(c->n_heads);
  for (int l = 0; l < c->n_heads; ++l) {
    if ((e = dev_alloc(c, &c->Wf[l], wf_frags)) != hipSuccess) return bail(e, "hipMalloc(W)");
    if ((e = dev_alloc(c, &c->gamma[l], (size_t)c->d)) != hipSuccess) return bail(e, "hipMalloc(gamma)");
    if ((e = dev_alloc(c, &c->beta[l], (size_t)c->d)) != hipSuccess) return bail(e, "hipMalloc(beta)");
    const unsigned blocks = (unsigned)((wf_frags + 255) / 256);
    if (c->dtype == EH_BF16)
      hipLaunchKernelGGL((repack_w_kernel<DtBf16>), dim3(blocks), dim3(256), 0, 0, cfg->W[l], c->V,
                         c->d, c->VT, c->KS, c->Wf[l]);
    else
      hipLaunchKernelGGL((repack_w_kernel<DtF32>), dim3(blocks), dim3(256), 0, 0, cfg->W[l], c->V,
                         c->d, c->VT, c->KS, c->Wf[l]);
    if ((e = hipGetLastError()) != hipSuccess) return bail(e, "repack launch");
    if ((e = hipMemcpy(c->gamma[l], cfg->gamma[l], sizeof(float) * c->d, hipMemcpyDeviceToDevice)) != hipSuccess)
      return bail(e, "copy gamma");
    if ((e = hipMemcpy(c->beta[l], cfg->beta[l], sizeof(float) * c->d, hipMemcpyDeviceToDevice)) != hipSuccess)
      return bail(e, "copy beta");
    if (cfg->bias) {
      if ((e = dev_alloc(c, &c->bias[l], (size_t)Vp)) != hipSuccess) return bail(e, "hipMalloc(bias)");
      if ((e = hipMemset(c->bias[l], 0, sizeof(float) * Vp)) != hipSuccess) return bail(e, "memset bias");
      if ((e = hipMemcpy(c->bias[l], cfg->bias[l], sizeof(float) * c->V, hipMemcpyDeviceToDevice)) != hipSuccess)
        return bail(e, "copy bias");
    }
  }
  // the kernels read whole groups of token blocks: up to kMaxNB (stream kernel) or 4 waves x 8
  // blocks (batched kernel) starting inside the padded rows, so 32 zero blocks follow them
  const size_t y_frags = (size_t)(c->R_pad_max / 16 + 32) * c->KS * kWave;
  if ((e = dev_alloc(c, &c->yf, y_frags)) != hipSuccess) return bail(e, "hipMalloc(y)");
  if ((e = hipMemset(c->yf, 0, y_frags * sizeof(frag_t))) != hipSuccess) return bail(e, "memset y");
  if ((e = dev_alloc(c, &c->partials, (size_t)kStreamGrid * c->R_pad_max)) != hipSuccess)
    return bail(e, "hipMalloc(partials)");
  if ((e = dev_alloc(c, &c->ws_H, (size_t)c->max_rows)) != hipSuccess) return bail(e, "hipMalloc(ws)");
  if ((e = dev_alloc(c, &c->ws_lse, (size_t)c->max_rows)) != hipSuccess) return bail(e, "hipMalloc(ws)");
  if ((e = dev_alloc(c, &c->ws_argmax, (size_t)c->max_rows)) != hipSuccess) return bail(e, "hipMalloc(ws)");
  for (int i = 0; i < 2; ++i) {
    if ((e = dev_alloc(c, &c->active[i], (size_t)c->max_rows)) != hipSuccess) return bail(e, "hipMalloc(ws)");
    if ((e = dev_alloc(c, &c->n_active[i], (size_t)4)) != hipSuccess) return bail(e, "hipMalloc(ws)");
  }
  {
    // device-side tables for the persistent decode kernel
    const size_t np = (size_t)c->n_heads;
    if ((e = dev_alloc(c, &c->d_Wf, np)) != hipSuccess) return bail(e, "hipMalloc(tables)");
    if ((e = dev_alloc(c, &c->d_gamma, np)) != hipSuccess) return bail(e, "hipMalloc(tables)");
    if ((e = dev_alloc(c, &c->d_beta, np)) != hipSuccess) return bail(e, "hipMalloc(tables)");
    if ((e = dev_alloc(c, &c->d_tau, np)) != hipSuccess) return bail(e, "hipMalloc(tables)");
    if ((e = hipMemcpy(c->d_Wf, c->Wf.data(), np * sizeof(void*), hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "copy tables");
    if ((e = hipMemcpy(c->d_gamma, c->gamma.data(), np * sizeof(void*), hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "copy tables");
    if ((e = hipMemcpy(c->d_beta, c->beta.data(), np * sizeof(void*), hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "copy tables");
    if ((e = hipMemcpy(c->d_tau, c->tau.data(), np * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "copy tables");
    if (cfg->bias) {
      if ((e = dev_alloc(c, &c->d_bias, np)) != hipSuccess) return bail(e, "hipMalloc(tables)");
      if ((e = hipMemcpy(c->d_bias, c->bias.data(), np * sizeof(void*), hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "copy tables");
    }
    if ((e = decode_prepare(c)) != hipSuccess) return bail(e, "decode_prepare");
    if ((e = rows_prepare(c)) != hipSuccess) return bail(e, "rows_prepare");
    if (c->rows_grid > 0 && (c->max_rows > 16 || c->decode_grid == 0)) {
      // workspace of the persistent kernel for 17 .. 256 rows: one activation buffer per head (plus
      // the blocks a wave may read past the last live one), two sets of partial statistics
      const int rmax = std::min(c->R_pad_max, kRowsMax);
      c->rows_y_stride = (long long)(rmax / 16 + 32) * c->KS * kWave;
      c->rows_ctl_ints = rows_control_ints(c->n_heads);
      if ((e = dev_alloc(c, &c->rows_y, (size_t)c->n_heads * c->rows_y_stride)) != hipSuccess) return bail(e, "hipMalloc(rows)");
      if ((e = hipMemset(c->rows_y, 0, (size_t)c->n_heads * c->rows_y_stride * sizeof(frag_t))) != hipSuccess) return bail(e, "memset rows");
      if ((e = dev_alloc(c, &c->rows_part4, (size_t)2 * c->rows_grid * rmax)) != hipSuccess) return bail(e, "hipMalloc(rows)");
      if ((e = dev_alloc(c, &c->rows_parti, (size_t)2 * c->rows_grid * rmax)) != hipSuccess) return bail(e, "hipMalloc(rows)");
      if ((e = dev_alloc(c, &c->rows_ctl, (size_t)c->rows_ctl_ints)) != hipSuccess) return bail(e, "hipMalloc(rows)");
      c->rows_vctl_ints = rows_control_ints(1);
      if ((e = dev_alloc(c, &c->rows_vctl, (size_t)2 * c->rows_vctl_ints)) != hipSuccess) return bail(e, "hipMalloc(rows)");
      if ((e = hipMemset(c->rows_vctl, 0, (size_t)2 * c->rows_vctl_ints * sizeof(int))) != hipSuccess) return bail(e, "memset rows");
    } else {
      c->rows_grid = 0;
    }
    {
      hipDeviceProp_t prop;
      if ((e = hipGetDeviceProperties(&prop, c->device)) != hipSuccess) return bail(e, "device properties");
      c->num_cu = prop.multiProcessorCount;
#ifdef EH_DIAGNOSTICS
      const char* env = getenv("EH_DISABLE_GEMM");   // force the simple streaming kernel
      c->use_gemm = !(env && env[0] == '1');
#endif
    }
    // the status word both persistent kernels report a given-up wait in (read by eh_check)
    if ((e = dev_alloc(c, &c->dec_status, (size_t)4)) != hipSuccess) return bail(e, "hipMalloc(status)");
    if ((e = hipMemset(c->dec_status, 0, 16)) != hipSuccess) return bail(e, "memset");
    if (c->decode_grid > 0) {
      const size_t nrec = 2 * np * c->decode_grid * 16 * 5;
      if ((e = dev_alloc(c, &c->dec_records, nrec)) != hipSuccess) return bail(e, "hipMalloc(decode)");
      if ((e = hipMemset(c->dec_records, 0, nrec * sizeof(unsigned long long))) != hipSuccess) return bail(e, "memset");
      if ((e = dev_alloc(c, &c->dec_trace, np * 16 + 4 * (size_t)c->decode_grid)) != hipSuccess) return bail(e, "hipMalloc(decode)");
      if ((e = hipMemset(c->dec_trace, 0, (np * 16 + 4 * (size_t)c->decode_grid) * sizeof(unsigned long long))) != hipSuccess) return bail(e, "memset");
    }
  }
  if ((e = hipDeviceSynchronize()) != hipSuccess) return bail(e, "eh_create sync");
  *out = c;
  return EH_OK;
}

eh_status eh_destroy(eh_ctx* ctx) {
  if (!ctx) return EH_ERR_NULL;
  DeviceGuard guard(ctx->device);
  (void)hipDeviceSynchronize();
  free_all(ctx);
  delete ctx;
  return EH_OK;
}

eh_status eh_eval(eh_ctx* ctx, int32_t head, const void* h, int64_t h_row_stride,
                  const int32_t* row_idx, const int32_t* n_rows_dev, int32_t n_rows, float* H,
                  float* lse, int32_t* argmax, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (head < 0 || head >= ctx->n_heads) return fail(ctx, EH_ERR_RANGE, "head out of range");
  if (n_rows == 0) return EH_OK;
  if (!h) return fail(ctx, EH_ERR_NULL, "h is NULL");
  eh_status st = check_rows(ctx, h, h_row_stride, n_rows);
  if (st != EH_OK) return st;
  DeviceGuard guard(ctx->device);
  if (use_decode(ctx, n_rows)) {
    DecodeParams p = decode_base(ctx);
    p.h = h; p.layer_stride = 0; p.row_stride = h_row_stride; p.row_idx = row_idx;
    p.n_rows_dev = n_rows_dev; p.n_rows = n_rows; p.l0 = 0; p.l1 = 1; p.decide = 0;
    // evaluation mode addresses one head: shift the tables instead of the layer stride
    p.Wf += head; p.gamma += head; p.beta += head; if (p.bias) p.bias += head;
    p.records += (size_t)head * ctx->decode_grid * 16 * 5;
    p.H = H; p.lse = lse; p.argmax = argmax;
    EH_HIP(ctx, decode_launch(ctx, p, (hipStream_t)stream));
    return EH_OK;
  }
  return run_head<false>(ctx, head, h, h_row_stride, row_idx, n_rows_dev, n_rows, H, lse, argmax,
                         (hipStream_t)stream);
}

eh_status eh_eval_noalloc(eh_ctx* ctx, int32_t head, const void* h, int64_t h_row_stride,
                          const int32_t* row_idx, const int32_t* n_rows_dev, int32_t n_rows, float* H,
                          float* lse, int32_t* argmax, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (head < 0 || head >= ctx->n_heads) return fail(ctx, EH_ERR_RANGE, "head out of range");
  if (n_rows < 0) return fail(ctx, EH_ERR_SHAPE, "n_rows is negative");
  if (n_rows == 0) return EH_OK;
  if (!h) return fail(ctx, EH_ERR_NULL, "h is NULL");
  if (h_row_stride < ctx->d) return fail(ctx, EH_ERR_SHAPE, "row stride smaller than d");
  const int esz = ctx->dtype == EH_BF16 ? 2 : 4;
  if (!aligned16(h) || (h_row_stride * esz) % 16 != 0)
    return fail(ctx, EH_ERR_SHAPE, "hidden rows must be 16-byte aligned");
  // layout of the static array for this call: activations of the rows (padded to blocks of 32,
  // plus the 32 blocks of 16 the batched kernels may read beyond them), then one partial
  // statistics record per (workgroup, row)
  const size_t R_pad = ((size_t)n_rows + 31) & ~(size_t)31;
  const size_t y_bytes = (R_pad / 16 + 32) * (size_t)ctx->KS * kWave * sizeof(frag_t);
  const size_t part_off = (y_bytes + 255) & ~(size_t)255;
  const size_t need = part_off + (size_t)kStreamGrid * R_pad * sizeof(Stats);
  if ((size_t)n_rows > ((size_t)1 << 20) || need > kNoAllocScratchBytes)
    return fail(ctx, EH_ERR_WORKSPACE,
                "n_rows rows of d elements need " + std::to_string(need) + " bytes of workspace; the static one holds " +
                    std::to_string(kNoAllocScratchBytes));
  if (!ctx->static_scratch) return fail(ctx, EH_ERR_HIP, "the static workspace has no device address");
  DeviceGuard guard(ctx->device);
  unsigned char* base = (unsigned char*)ctx->static_scratch;
  return run_head<false>(ctx, head, h, h_row_stride, row_idx, n_rows_dev, n_rows, H, lse, argmax,
                         (hipStream_t)stream, (frag_t*)base, (Stats*)(base + part_off));
}

namespace {

// eh_eval_heads and eh_eval_heads_metrics.  `metrics`: also the maximum probability and the
// difference of the two largest probabilities (either output may be NULL).
// The many-heads workspace: per head, activations for max_rows rows (plus the zero blocks the
// batched kernel may read past them), one set of partial statistics and one of second largest
// logits.  Grow-only, kept by the context; the old one may still be in use on a stream.
eh_status ensure_mh(eh_ctx* ctx, int n_heads_needed) {
  if (ctx->mh_heads >= n_heads_needed) return EH_OK;
  const size_t y_stride = (size_t)(ctx->R_pad_max / 16 + 32) * ctx->KS * kWave;
  const size_t part_stride = (size_t)kStreamGrid * ctx->R_pad_max;
  EH_HIP(ctx, hipDeviceSynchronize());
  eh::frag_t* y = nullptr;
  eh::Stats* pt = nullptr;
  float* sec = nullptr;
  hipError_t e = dev_alloc(ctx, &y, y_stride * n_heads_needed);
  if (e == hipSuccess) e = dev_alloc(ctx, &pt, part_stride * n_heads_needed);
  if (e == hipSuccess) e = dev_alloc(ctx, &sec, part_stride * n_heads_needed);
  if (e == hipSuccess) e = hipMemset(y, 0, y_stride * n_heads_needed * sizeof(frag_t));
  EH_HIP(ctx, e);
  ctx->mh_yf = y;
  ctx->mh_partials = pt;
  ctx->mh_second = sec;
  ctx->mh_heads = n_heads_needed;
  return EH_OK;
}

eh_status eval_heads_impl(eh_ctx* ctx, int32_t head0, int32_t n_heads_eval, const void* h_layers,
                          int64_t layer_stride, int64_t row_stride, int32_t n_rows, float* H, float* lse,
                          int32_t* argmax, bool metrics, float* max_prob, float* margin, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (n_heads_eval < 0 || head0 < 0 || head0 + n_heads_eval > ctx->n_heads)
    return fail(ctx, EH_ERR_RANGE, "heads out of range");
  if (metrics && (ctx->dtype != EH_BF16 || !ctx->bias.empty()))
    return fail(ctx, EH_ERR_DTYPE, "the extra confidence metrics need bf16 heads without a bias vector");
  if (n_rows == 0 || n_heads_eval == 0) return EH_OK;
  if (!h_layers) return fail(ctx, EH_ERR_NULL, "h_layers is NULL");
  eh_status st = check_rows(ctx, h_layers, row_stride, n_rows);
  if (st != EH_OK) return st;
  const int esz = ctx->dtype == EH_BF16 ? 2 : 4;
  if ((layer_stride * esz) % 16 != 0) return fail(ctx, EH_ERR_SHAPE, "hidden rows must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const bool batched =
      ctx->dtype == EH_BF16 && ctx->bias.empty() && ((ctx->use_gemm && n_rows > 16) || metrics);
  if (!batched) {
    // shapes the many-heads kernels do not cover: one head after the other
    for (int l = 0; l < n_heads_eval; ++l) {
      st = eh_eval(ctx, head0 + l, (const char*)h_layers + (int64_t)l * layer_stride * esz, row_stride,
                   nullptr, nullptr, n_rows, H ? H + (int64_t)l * n_rows : nullptr,
                   lse ? lse + (int64_t)l * n_rows : nullptr,
                   argmax ? argmax + (int64_t)l * n_rows : nullptr, stream);
      if (st != EH_OK) return st;
    }
    return EH_OK;
  }
  DeviceGuard guard(ctx->device);
  // per head: activations for max_rows rows (plus the zero blocks the kernel may read past
  // them), one set of partial statistics and one of second largest logits
  const size_t y_stride = (size_t)(ctx->R_pad_max / 16 + 32) * ctx->KS * kWave;
  const size_t part_stride = (size_t)kStreamGrid * ctx->R_pad_max;
  st = ensure_mh(ctx, n_heads_eval);
  if (st != EH_OK) return st;
  const int R_pad = (n_rows + 31) & ~31;
  hipLaunchKernelGGL((ln_pack_heads_kernel<DtBf16, 32>), dim3(R_pad, n_heads_eval), dim3(kLnThreads), 0, s, h_layers,
                     layer_stride, row_stride, n_rows, R_pad, ctx->d, ctx->KS,
                     (const float* const*)(ctx->d_gamma + head0), (const float* const*)(ctx->d_beta + head0),
                     ctx->eps, ctx->mh_yf, (int64_t)y_stride);
  int n_parts = 0;
  EH_HIP(ctx, gemm32_launch_heads(ctx, head0, n_heads_eval, nullptr, n_rows, false, ctx->mh_yf, (long long)y_stride,
                                  ctx->mh_partials, metrics ? ctx->mh_second : nullptr, (long long)part_stride,
                                  &n_parts, s));
  if (metrics)
    hipLaunchKernelGGL(finalize_metrics_kernel, dim3(n_rows, n_heads_eval), dim3(64), 0, s, ctx->mh_partials,
                       ctx->mh_second, n_parts, R_pad, n_rows, H, lse, argmax, max_prob, margin,
                       (int64_t)part_stride, (int64_t)n_rows);
  else
    hipLaunchKernelGGL(finalize_kernel, dim3(n_rows, n_heads_eval), dim3(64), 0, s, ctx->mh_partials, n_parts,
                       R_pad, (const int*)nullptr, n_rows, H, lse, argmax, (int64_t)part_stride,
                       (int64_t)n_rows);
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

}  // namespace

eh_status eh_eval_heads(eh_ctx* ctx, int32_t head0, int32_t n_heads_eval, const void* h_layers,
                        int64_t layer_stride, int64_t row_stride, int32_t n_rows, float* H, float* lse,
                        int32_t* argmax, void* stream) {
  return eval_heads_impl(ctx, head0, n_heads_eval, h_layers, layer_stride, row_stride, n_rows, H, lse, argmax,
                         false, nullptr, nullptr, stream);
}

eh_status eh_eval_heads_metrics(eh_ctx* ctx, int32_t head0, int32_t n_heads_eval, const void* h_layers,
                                int64_t layer_stride, int64_t row_stride, int32_t n_rows, float* H, float* lse,
                                int32_t* argmax, float* max_prob, float* margin, void* stream) {
  return eval_heads_impl(ctx, head0, n_heads_eval, h_layers, layer_stride, row_stride, n_rows, H, lse, argmax,
                         true, max_prob, margin, stream);
}

eh_status eh_exit_decide(eh_ctx* ctx, int32_t head, const float* H, const int32_t* argmax,
                         const int32_t* row_idx, const int32_t* n_rows_dev, int32_t n_rows,
                         int32_t* exit_layer, int32_t* token, int32_t* active_idx_out,
                         int32_t* n_active_out, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (head < 0 || head >= ctx->n_heads) return fail(ctx, EH_ERR_RANGE, "head out of range");
  if (n_rows < 0 || n_rows > ctx->max_rows) return fail(ctx, EH_ERR_WORKSPACE, "n_rows outside [0, max_rows]");
  if (!H || !argmax || !exit_layer || !token || !active_idx_out || !n_active_out)
    return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  if (active_idx_out == row_idx) return fail(ctx, EH_ERR_RANGE, "active_idx_out must not alias row_idx");
  DeviceGuard guard(ctx->device);
  const float tau = ctx->tau[head];
  hipLaunchKernelGGL(decide_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, H, argmax, row_idx,
                     n_rows_dev, n_rows, tau, head == ctx->n_heads - 1 ? 1 : 0, head, exit_layer, token,
                     active_idx_out, n_active_out, (float*)nullptr, (unsigned long long*)nullptr);
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

eh_status eh_cascade(eh_ctx* ctx, const void* h_layers, int64_t layer_stride, int64_t row_stride,
                     int32_t n_rows, int32_t* exit_layer, int32_t* token, float* H_out,
                     int64_t* n_evals_out, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (n_rows == 0) return EH_OK;
  if (!h_layers || !exit_layer || !token) return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  eh_status st = check_rows(ctx, h_layers, row_stride, n_rows);
  if (st != EH_OK) return st;
  const int esz = ctx->dtype == EH_BF16 ? 2 : 4;
  if (ctx->n_heads > 1 && (layer_stride * esz) % 16 != 0)
    return fail(ctx, EH_ERR_SHAPE, "layer stride must keep rows 16-byte aligned");
  DeviceGuard guard(ctx->device);
  hipStream_t s = (hipStream_t)stream;
  if (use_decode(ctx, n_rows)) {
    DecodeParams p = decode_base(ctx);
    p.h = h_layers; p.layer_stride = layer_stride; p.row_stride = row_stride;
    p.n_rows = n_rows; p.l0 = 0; p.l1 = ctx->n_heads; p.decide = 1;
    p.exit_layer = exit_layer; p.token = token; p.H_out = H_out;
    p.n_evals = (unsigned long long*)n_evals_out;
    EH_HIP(ctx, decode_launch(ctx, p, s));
    return EH_OK;
  }
  if (use_rows(ctx, n_rows)) {
    // one persistent launch for the whole cascade
    RowsParams p = rows_base(ctx, n_rows);
    p.h = h_layers; p.layer_stride = layer_stride; p.row_stride = row_stride;
    p.l0 = 0; p.l1 = ctx->n_heads; p.mode = 0; p.argmax_only = 0;
    p.exit_layer = exit_layer; p.token = token; p.H_out = H_out;
    p.n_evals = (unsigned long long*)n_evals_out;
    EH_HIP(ctx, rows_launch(ctx, p, s));
    return EH_OK;
  }
  if (H_out) {
    const int64_t n = (int64_t)ctx->n_heads * n_rows;
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, H_out, n, NAN);
  }
  if (ctx->bias.empty() && ctx->use_gemm) {
    // Two launches per head: the batched projection, then one kernel that merges the partial
    // statistics, applies the exit rule, appends the rows that go on to the next head's list
    // and writes their LayerNorm for the next head.  Three live-row counters rotate: head l
    // reads counter l%3, fills (l+1)%3 and clears (l+2)%3.
    const bool bf = ctx->dtype == EH_BF16;
    const int RB = bf ? 32 : 16;
    const int R_pad = (n_rows + RB - 1) / RB * RB;
    int* cnt = ctx->n_active[0];
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, s, cnt, (int64_t)3, 0);
    {
      dim3 g(R_pad), b(kLnThreads);
      if (bf)
        hipLaunchKernelGGL((ln_pack_kernel<DtBf16, 32>), g, b, 0, s, h_layers, row_stride, (const int*)nullptr,
                           (const int*)nullptr, n_rows, R_pad, ctx->d, ctx->KS, ctx->gamma[0], ctx->beta[0],
                           ctx->eps, ctx->yf);
      else
        hipLaunchKernelGGL((ln_pack_kernel<DtF32, 16>), g, b, 0, s, h_layers, row_stride, (const int*)nullptr,
                           (const int*)nullptr, n_rows, R_pad, ctx->d, ctx->KS, ctx->gamma[0], ctx->beta[0],
                           ctx->eps, ctx->yf);
    }
    for (int l = 0; l < ctx->n_heads; ++l) {
      const int last = l == ctx->n_heads - 1 ? 1 : 0;
      const int* idx = l == 0 ? nullptr : ctx->active[l & 1];
      const int* live = l == 0 ? nullptr : cnt + l % 3;
      int n_parts = 0;
      if (bf) EH_HIP(ctx, gemm32_launch(ctx, l, live, n_rows, false, ctx->yf, ctx->partials, nullptr, &n_parts, s));
      else EH_HIP(ctx, gemm_launch(ctx, l, live, n_rows, false, ctx->yf, ctx->partials, &n_parts, s));
      const void* hn = last ? nullptr : (const char*)h_layers + (int64_t)(l + 1) * layer_stride * esz;
      const float* gn = last ? nullptr : ctx->gamma[l + 1];
      const float* bn = last ? nullptr : ctx->beta[l + 1];
      float* Hl = H_out ? H_out + (int64_t)l * n_rows : nullptr;
#define EH_POST(DT, RBV)                                                                              \
  hipLaunchKernelGGL((cascade_post_kernel<DT, RBV>), dim3(n_rows), dim3(kLnThreads), 0, s, ctx->partials, n_parts, \
                     R_pad, idx, live, n_rows, ctx->tau[l], last, l, exit_layer, token, Hl,            \
                     (unsigned long long*)n_evals_out, ctx->active[(l + 1) & 1], cnt + (l + 1) % 3,    \
                     cnt + (l + 2) % 3, hn, row_stride, ctx->d, ctx->KS, gn, bn, ctx->eps, ctx->yf)
      if (bf) EH_POST(DtBf16, 32);
      else EH_POST(DtF32, 16);
#undef EH_POST
    }
    EH_HIP(ctx, hipGetLastError());
    return EH_OK;
  }
  for (int l = 0; l < ctx->n_heads; ++l) {
    const int* idx = l == 0 ? nullptr : ctx->active[(l - 1) & 1];
    const int* cnt = l == 0 ? nullptr : ctx->n_active[(l - 1) & 1];
    const void* hl = (const char*)h_layers + (int64_t)l * layer_stride * esz;
    st = run_head<false>(ctx, l, hl, row_stride, idx, cnt, n_rows, ctx->ws_H, ctx->ws_lse,
                         ctx->ws_argmax, s);
    if (st != EH_OK) return st;
    hipLaunchKernelGGL(decide_kernel, dim3(1), dim3(256), 0, s, ctx->ws_H, ctx->ws_argmax, idx, cnt,
                       n_rows, ctx->tau[l], l == ctx->n_heads - 1 ? 1 : 0, l, exit_layer, token,
                       ctx->active[l & 1], ctx->n_active[l & 1],
                       H_out ? H_out + (int64_t)l * n_rows : nullptr, (unsigned long long*)n_evals_out);
  }
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

eh_status dssd_verify(eh_ctx* ctx, const void* f_final, const int32_t* draft, const int32_t* draft_len,
                      int32_t B, int32_t k, int32_t* accepted, int32_t* next_token, int32_t* target,
                      void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (B < 0 || k < 0) return fail(ctx, EH_ERR_SHAPE, "B and k must be non-negative");
  if (B == 0) return EH_OK;
  if (!f_final || !accepted || !next_token || (k > 0 && !draft))
    return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  const int64_t rows = (int64_t)B * (k + 1);
  if (rows > ctx->max_rows) return fail(ctx, EH_ERR_WORKSPACE, "B*(k+1) exceeds max_rows");
  eh_status st = check_rows(ctx, f_final, ctx->d, (int)rows);
  if (st != EH_OK) return st;
  DeviceGuard guard(ctx->device);
  hipStream_t s = (hipStream_t)stream;
  const bool bf = ctx->dtype == EH_BF16;
  if (use_rows(ctx, rows)) {
    // one persistent launch: LayerNorm, argmax-only projection, merge and prefix walk
    RowsParams p = rows_base(ctx, (int)rows);
    p.h = f_final; p.layer_stride = 0; p.row_stride = ctx->d;
    p.l0 = ctx->n_heads - 1; p.l1 = ctx->n_heads; p.mode = 1; p.argmax_only = 1;
    p.n_stream = ctx->rows_grid;  // a verification has no serving workgroups: all stream, then all merge
    // no preset launch in front of a verification: it runs on one of two control blocks in turn and
    // clears the other for the call after it (calls on a context are serialised)
    p.ctl = ctx->rows_vctl + (size_t)(ctx->rows_vturn & 1u) * ctx->rows_vctl_ints;
    p.ctl_next = ctx->rows_vctl + (size_t)((ctx->rows_vturn + 1u) & 1u) * ctx->rows_vctl_ints;
    p.n_ctl_next = ctx->rows_vctl_ints;
    ++ctx->rows_vturn;
    p.draft = draft; p.draft_len = draft_len; p.B = B; p.k = k;
    p.accepted = accepted; p.next_token = next_token; p.target = target;
    EH_HIP(ctx, rows_launch(ctx, p, s));
    return EH_OK;
  }
  if (ctx->bias.empty() && ctx->use_gemm && rows > 16 && (size_t)(k + 1) * sizeof(int) <= 48 * 1024) {
    // three launches: LayerNorm, argmax-only projection, then one kernel that merges the
    // partial argmaxes of a row's k+1 positions and walks the prefix
    const int RB = bf ? 32 : 16;
    const int R_pad = (int)((rows + RB - 1) / RB * RB);
    const int fin = ctx->n_heads - 1;
    dim3 g(R_pad), b(kLnThreads);
    if (bf)
      hipLaunchKernelGGL((ln_pack_kernel<DtBf16, 32>), g, b, 0, s, f_final, (int64_t)ctx->d, (const int*)nullptr,
                         (const int*)nullptr, (int)rows, R_pad, ctx->d, ctx->KS, ctx->gamma[fin], ctx->beta[fin],
                         ctx->eps, ctx->yf);
    else
      hipLaunchKernelGGL((ln_pack_kernel<DtF32, 16>), g, b, 0, s, f_final, (int64_t)ctx->d, (const int*)nullptr,
                         (const int*)nullptr, (int)rows, R_pad, ctx->d, ctx->KS, ctx->gamma[fin], ctx->beta[fin],
                         ctx->eps, ctx->yf);
    int n_parts = 0;
    if (bf) EH_HIP(ctx, gemm32_launch(ctx, fin, nullptr, (int)rows, true, ctx->yf, ctx->partials, nullptr, &n_parts, s));
    else EH_HIP(ctx, gemm_launch(ctx, fin, nullptr, (int)rows, true, ctx->yf, ctx->partials, &n_parts, s));
    hipLaunchKernelGGL(verify_post_kernel, dim3(B), dim3(256), (size_t)(k + 1) * sizeof(int), s, ctx->partials,
                       n_parts, R_pad, draft, draft_len, k, target, accepted, next_token);
    EH_HIP(ctx, hipGetLastError());
    return EH_OK;
  }
  int* tgt = target ? target : ctx->ws_argmax;
  st = run_head<true>(ctx, ctx->n_heads - 1, f_final, ctx->d, nullptr, nullptr, (int)rows, nullptr,
                      nullptr, tgt, s);
  if (st != EH_OK) return st;
  hipLaunchKernelGGL(verify_compare_kernel, dim3((B + 63) / 64), dim3(64), 0, s, draft, draft_len, tgt, B,
                     k, accepted, next_token);
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

eh_status dssd_draft(eh_ctx* ctx, const void* h_positions, int64_t pos_stride, int64_t layer_stride,
                     int32_t n_positions, int32_t limit, int32_t eos_token, int32_t* draft, int32_t* draft_len,
                     int32_t* exit_layers, int32_t* stop_reason, int32_t* fallback_token, int64_t* n_evals_out,
                     void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (limit < 0 || n_positions < 0) return fail(ctx, EH_ERR_SHAPE, "limit and n_positions must be non-negative");
  if (!draft_len || (limit > 0 && (!draft || !exit_layers))) return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  if (n_positions > 0 && limit > 0 && !h_positions) return fail(ctx, EH_ERR_NULL, "h_positions is NULL");
  const bool by_rows = ctx->decode_grid <= 0 && use_rows(ctx, 1);  // hidden sizes above the decode kernel's
  if (ctx->decode_grid <= 0 && !by_rows)
    return fail(ctx, EH_ERR_DTYPE, "drafting needs a single-launch cascade kernel (bf16 or fp32 heads without a bias "
                                   "vector; fp32 up to d = 1024)");
  if (ctx->n_heads < 2) return fail(ctx, EH_ERR_RANGE, "drafting needs at least one exit head besides the model's");
  const int esz = ctx->dtype == EH_BF16 ? 2 : 4;
  const int steps = n_positions < limit ? n_positions : limit;
  if (steps > 0) {
    eh_status st = check_rows(ctx, h_positions, ctx->d, 1);
    if (st != EH_OK) return st;
    if ((layer_stride * esz) % 16 != 0 || (pos_stride * esz) % 16 != 0)
      return fail(ctx, EH_ERR_SHAPE, "strides must keep rows 16-byte aligned");
  }
  DeviceGuard guard(ctx->device);
  hipStream_t s = (hipStream_t)stream;
  int* state = ctx->n_active[1];     // {live, length, reason, fallback token}
  int* ex = ctx->active[0];          // the current position's exit layer and token
  int* tk = ctx->active[1];
  hipLaunchKernelGGL(draft_init_kernel, dim3(1), dim3(64), 0, s, state, limit, exit_layers);
  for (int t = 0; t < steps && by_rows; ++t) {
    RowsParams p = rows_base(ctx, 1);
    p.h = (const char*)h_positions + (int64_t)t * pos_stride * esz;
    p.layer_stride = layer_stride;
    p.row_stride = ctx->d;
    p.l0 = 0; p.l1 = ctx->n_heads; p.mode = 0; p.argmax_only = 0;
    p.live = state;  // 1 while drafting, 0 once it has stopped: both launches then return at once
    p.exit_layer = ex; p.token = tk; p.H_out = nullptr;
    p.n_evals = (unsigned long long*)n_evals_out;
    EH_HIP(ctx, rows_launch(ctx, p, s));
    hipLaunchKernelGGL(draft_step_kernel, dim3(1), dim3(1), 0, s, state, ex, tk, ctx->n_heads - 1, limit, eos_token,
                       draft, exit_layers);
  }
  for (int t = 0; t < steps && !by_rows; ++t) {
    DecodeParams p = decode_base(ctx);
    p.h = (const char*)h_positions + (int64_t)t * pos_stride * esz;
    p.layer_stride = layer_stride;
    p.row_stride = ctx->d;
    p.n_rows = 1;
    p.n_rows_dev = state;  // 1 while drafting, 0 once it has stopped: the launch then returns at once
    p.l0 = 0;
    p.l1 = ctx->n_heads;
    p.decide = 1;
    p.exit_layer = ex;
    p.token = tk;
    p.H_out = nullptr;
    p.n_evals = (unsigned long long*)n_evals_out;
    EH_HIP(ctx, decode_launch(ctx, p, s));
    hipLaunchKernelGGL(draft_step_kernel, dim3(1), dim3(1), 0, s, state, ex, tk, ctx->n_heads - 1, limit, eos_token,
                       draft, exit_layers);
  }
  hipLaunchKernelGGL(draft_finish_kernel, dim3(1), dim3(1), 0, s, state, draft_len, stop_reason, fallback_token);
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

eh_status dssd_tally(eh_ctx* ctx, const int32_t* draft_len, const int32_t* accepted, int32_t B, int32_t k,
                     const int32_t* exit_layers, int64_t* counters, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (B < 0 || k < 0) return fail(ctx, EH_ERR_SHAPE, "B and k must be non-negative");
  if (!counters || (B > 0 && !accepted)) return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  if (B == 0) return EH_OK;
  DeviceGuard guard(ctx->device);
  hipLaunchKernelGGL(tally_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, draft_len, accepted, B, k, exit_layers,
                     (unsigned long long*)counters);
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

eh_status eh_head_losses(eh_ctx* ctx, int32_t head, const void* h_head, int64_t row_stride_head,
                         const void* h_model, int64_t row_stride_model, const int32_t* labels, int32_t n_rows,
                         float alpha, float* kl, float* ce, float* loss, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (head < 0 || head >= ctx->n_heads) return fail(ctx, EH_ERR_RANGE, "head out of range");
  if (ctx->dtype != EH_BF16 || !ctx->bias.empty())
    return fail(ctx, EH_ERR_DTYPE, "the fused objectives need bf16 heads without a bias vector");
  if (n_rows <= 0) return fail(ctx, EH_ERR_SHAPE, "the mean over an empty sequence is undefined");
  if (!h_head || !h_model || !loss) return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  eh_status st = check_rows(ctx, h_head, row_stride_head, n_rows);
  if (st == EH_OK) st = check_rows(ctx, h_model, row_stride_model, n_rows);
  if (st != EH_OK) return st;
  DeviceGuard guard(ctx->device);
  hipStream_t s = (hipStream_t)stream;
  st = ensure_mh(ctx, 2);
  if (st != EH_OK) return st;
  if (!ctx->kl_partials) {
    EH_HIP(ctx, dev_alloc(ctx, &ctx->kl_partials, (size_t)kStreamGrid * ctx->R_pad_max));
    EH_HIP(ctx, dev_alloc(ctx, &ctx->kl_rows, (size_t)2 * ctx->R_pad_max));
  }
  const size_t y_stride = (size_t)(ctx->R_pad_max / 16 + 32) * ctx->KS * kWave;
  const int R_pad = (n_rows + 31) & ~31;
  const int fin = ctx->n_heads - 1;
  hipLaunchKernelGGL((ln_pack_kernel<DtBf16, 32>), dim3(R_pad), dim3(kLnThreads), 0, s, h_head, row_stride_head,
                     (const int*)nullptr, (const int*)nullptr, n_rows, R_pad, ctx->d, ctx->KS, ctx->gamma[head],
                     ctx->beta[head], ctx->eps, ctx->mh_yf);
  hipLaunchKernelGGL((ln_pack_kernel<DtBf16, 32>), dim3(R_pad), dim3(kLnThreads), 0, s, h_model, row_stride_model,
                     (const int*)nullptr, (const int*)nullptr, n_rows, R_pad, ctx->d, ctx->KS, ctx->gamma[fin],
                     ctx->beta[fin], ctx->eps, ctx->mh_yf + y_stride);
  int n_parts = 0;
  EH_HIP(ctx, gemm32_kl_launch(ctx, head, fin, n_rows, ctx->mh_yf, ctx->mh_yf + y_stride, labels, ctx->kl_partials,
                               &n_parts, s));
  hipLaunchKernelGGL(kl_finalize_kernel, dim3(n_rows), dim3(64), 0, s, ctx->kl_partials, n_parts, R_pad, n_rows,
                     ctx->V, ctx->kl_rows, kl, ce);
  hipLaunchKernelGGL(kl_mean_kernel, dim3(1), dim3(256), 0, s, ctx->kl_rows, R_pad, n_rows, alpha, loss);
  EH_HIP(ctx, hipGetLastError());
  return EH_OK;
}

eh_status eh_calibrate(eh_ctx* ctx, const float* H, const int32_t* pred, const int32_t* ref, int64_t M,
                       const double* eps, int32_t n_eps, float* tau_out, int64_t* n_exit_out, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (n_eps < 0 || n_eps > 64) return fail(ctx, EH_ERR_RANGE, "n_eps outside [0, 64]");
  if (M < 0 || M >= ((int64_t)1 << 31)) return fail(ctx, EH_ERR_SHAPE, "M outside [0, 2^31)");
  if (n_eps == 0) return EH_OK;
  if (!eps || !tau_out || (M > 0 && (!H || !pred || !ref))) return fail(ctx, EH_ERR_NULL, "a required pointer is NULL");
  for (int i = 0; i < n_eps; ++i)
    if (!(eps[i] >= 0.0 && eps[i] <= 1.0)) return fail(ctx, EH_ERR_RANGE, "epsilon outside [0, 1]");
  DeviceGuard guard(ctx->device);
  hipStream_t s = (hipStream_t)stream;
  if (M == 0) {
    hipLaunchKernelGGL(fill_f32_kernel, dim3(1), dim3(64), 0, s, tau_out, (int64_t)n_eps, -INFINITY);
    if (n_exit_out)
      hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(128), 0, s, (int*)n_exit_out, (int64_t)2 * n_eps, 0);
    EH_HIP(ctx, hipGetLastError());
    return EH_OK;
  }
  EH_HIP(ctx, calibrate_run(ctx->calib, H, pred, ref, M, eps, n_eps, tau_out, (long long*)n_exit_out, s));
  return EH_OK;
}

#ifdef EH_DIAGNOSTICS
// Diagnostics build: the 128 time-stamp words the last rows-kernel launch over n_heads heads left.
extern "C" eh_status eh_rows_trace(eh_ctx* ctx, int32_t n_heads, int32_t* host_out) {
  if (!ctx || !ctx->rows_ctl || !host_out) return EH_ERR_NULL;
  DeviceGuard guard(ctx->device);
  EH_HIP(ctx, hipDeviceSynchronize());
  const int* from = n_heads == 1 && ctx->rows_vturn > 0
                        ? ctx->rows_vctl + (size_t)((ctx->rows_vturn - 1u) & 1u) * ctx->rows_vctl_ints + ctx->rows_vctl_ints - 128
                        : ctx->rows_ctl + rows_control_ints(n_heads) - 128;
  EH_HIP(ctx, hipMemcpy(host_out, from, 128 * sizeof(int), hipMemcpyDeviceToHost));
  return EH_OK;
}
eh_status eh_decode_trace(eh_ctx* ctx, int32_t enable, uint64_t* host_out, int32_t n) {
  if (!ctx) return EH_ERR_NULL;
  if (!ctx->dec_trace) return fail(ctx, EH_ERR_RANGE, "this context has no decode kernel");
  DeviceGuard guard(ctx->device);
  if (host_out) {
    if (n < 0 || n > ctx->n_heads * 16 + 4 * ctx->decode_grid)
      return fail(ctx, EH_ERR_RANGE, "n outside [0, 16 * n_heads + 4 * workgroups]");
    EH_HIP(ctx, hipDeviceSynchronize());
    EH_HIP(ctx, hipMemcpy(host_out, ctx->dec_trace, sizeof(uint64_t) * n, hipMemcpyDeviceToHost));
  }
  ctx->dec_trace_on = enable ? 1 : 0;
  return EH_OK;
}
#endif

eh_status eh_check(eh_ctx* ctx, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  DeviceGuard guard(ctx->device);
  EH_HIP(ctx, hipStreamSynchronize((hipStream_t)stream));
  if (ctx->dec_status) {
    int flag = 0;
    EH_HIP(ctx, hipMemcpy(&flag, ctx->dec_status, sizeof(int), hipMemcpyDeviceToHost));
    if (flag != 0) {
      // report once and re-arm: the failed call's unfinished rows hold -1 / NaN
      EH_HIP(ctx, hipMemset(ctx->dec_status, 0, sizeof(int)));
      if (ctx->rows_vctl) EH_HIP(ctx, hipMemset(ctx->rows_vctl, 0, (size_t)2 * ctx->rows_vctl_ints * sizeof(int)));
      return fail(ctx, EH_ERR_HIP,
                  "the persistent kernel gave up waiting for another workgroup: the stream did not have the "
                  "device to itself (rows it did not finish hold -1 / NaN)");
    }
  }
  return EH_OK;
}

eh_status eh_set_spin_limit(eh_ctx* ctx, int32_t polls) {
  if (!ctx) return EH_ERR_NULL;
  if (polls < 0) return fail(ctx, EH_ERR_RANGE, "polls must be non-negative");
  ctx->spin_limit = polls;
  return EH_OK;
}

}  // extern "C"
