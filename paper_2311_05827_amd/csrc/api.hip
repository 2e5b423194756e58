// C ABI of libaccept: argument validation, size arithmetic, dispatch to the kernel
// launchers.  No device memory is allocated here and nothing is kept between calls.
#include <string.h>

#include <mutex>

#include "common.hpp"

using namespace accept;

namespace {

constexpr int64_t kMaxElems = int64_t(1) << 40;
constexpr int64_t kMaxChannels = int64_t(1) << 24;

// Scratch of accept_compress_noalloc: one array per GPU, part of the loaded code object, so it
// exists without any allocation call.  In host code the array's name is only a handle; the
// device address comes from hipGetSymbolAddress, once per device, and is what the kernels get.
constexpr size_t kScratchBytes = ACCEPT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the current device's scratch array (looked up on first use), or null.
void* scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

accept_status check_desc(const accept_desc* d) {
  if (!d) return ACCEPT_ERR_INVALID_ARG;
  if (d->scheme != ACCEPT_UNIFORM && d->scheme != ACCEPT_MBQ) return ACCEPT_ERR_INVALID_ARG;
  if (d->n < 1 || d->m < 1) return ACCEPT_ERR_INVALID_ARG;
  if (d->n > kMaxElems || d->m > kMaxElems || d->n > kMaxElems / d->m) return ACCEPT_ERR_INVALID_ARG;
  if (d->in_dtype != ACCEPT_F32 && d->in_dtype != ACCEPT_BF16) return ACCEPT_ERR_INVALID_ARG;
  if (d->out_dtype != ACCEPT_F32 && d->out_dtype != ACCEPT_BF16) return ACCEPT_ERR_INVALID_ARG;
  if (d->channels < 0 || d->channels > kMaxChannels) return ACCEPT_ERR_INVALID_ARG;
  if (d->layout != ACCEPT_LAYOUT_PACKED && d->layout != ACCEPT_LAYOUT_BATCH && d->layout != ACCEPT_LAYOUT_UNENCODED)
    return ACCEPT_ERR_INVALID_ARG;
  if (d->scheme == ACCEPT_UNIFORM) {
    if (d->bits < 2 || d->bits > 8) return ACCEPT_ERR_INVALID_ARG;
    if (d->layout == ACCEPT_LAYOUT_BATCH && 8 % d->bits != 0) return ACCEPT_ERR_INVALID_ARG;
    if (d->channels > 1 && d->m % d->channels != 0) return ACCEPT_ERR_INVALID_ARG;
    if (d->rounding != ACCEPT_ROUND_NEAREST_EVEN && d->rounding != ACCEPT_ROUND_STOCHASTIC)
      return ACCEPT_ERR_INVALID_ARG;
  } else {
    if (d->bits < 1 || d->bits > 8) return ACCEPT_ERR_INVALID_ARG;
    if (d->channels > 1) return ACCEPT_ERR_INVALID_ARG;
    if (d->layout == ACCEPT_LAYOUT_BATCH) return ACCEPT_ERR_INVALID_ARG;
    if (d->rounding != ACCEPT_ROUND_NEAREST_EVEN) return ACCEPT_ERR_INVALID_ARG;
    if (d->t < 0) return ACCEPT_ERR_INVALID_ARG;
  }
  return ACCEPT_OK;
}

accept_status finish_timer(StageTimer& tm, hipError_t launch_err, float* stage_ms, int* n_stages) {
  accept_status st = launch_err == hipSuccess && !tm.failed ? ACCEPT_OK : ACCEPT_ERR_HIP;
  if (tm.n > 0 && hipEventSynchronize(tm.ev[tm.n - 1]) != hipSuccess) st = ACCEPT_ERR_HIP;
  int stages = 0;
  if (st == ACCEPT_OK) {
    for (int i = 0; i + 1 < tm.n; ++i) {
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, tm.ev[i], tm.ev[i + 1]) != hipSuccess) { st = ACCEPT_ERR_HIP; break; }
      stage_ms[stages++] = ms;
    }
  }
  for (int i = 0; i < tm.n; ++i) (void)hipEventDestroy(tm.ev[i]);
  *n_stages = st == ACCEPT_OK ? stages : 0;
  return st;
}

accept_status do_compress(const accept_desc* d, const void* x, const float* alpha_prev, void* header, void* payload,
                          void* ws, void* stream, StageTimer* tm, hipError_t* launch_err) {
  *launch_err = hipSuccess;
  const accept_status st = check_desc(d);
  if (st != ACCEPT_OK) return st;
  if (!x || !header || !payload || !ws) return ACCEPT_ERR_INVALID_ARG;
  if (!aligned(x, 16) || !aligned(payload, 16) || !aligned(header, 4) || !aligned(ws, 256))
    return ACCEPT_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->scheme == ACCEPT_UNIFORM) {
    const UPlan p = make_uplan(*d);
    *launch_err = launch_uniform_compress(*d, p, x, header, payload, ws, s, tm);
  } else {
    if (!alpha_prev || !aligned(alpha_prev, 4)) return ACCEPT_ERR_INVALID_ARG;
    const MPlan p = make_mplan(*d);
    *launch_err = launch_mbq_compress(*d, p, x, alpha_prev, header, payload, ws, s, tm);
  }
  return *launch_err == hipSuccess ? ACCEPT_OK : ACCEPT_ERR_HIP;
}

accept_status do_decompress(const accept_desc* d, const void* header, const void* payload, void* xhat, void* stream,
                            StageTimer* tm, hipError_t* launch_err) {
  *launch_err = hipSuccess;
  const accept_status st = check_desc(d);
  if (st != ACCEPT_OK) return st;
  if (d->scheme == ACCEPT_UNIFORM && d->rounding == ACCEPT_ROUND_STOCHASTIC) {
    // rounding only affects compression; accepted here so that one descriptor serves both calls
  }
  if (!header || !payload || !xhat) return ACCEPT_ERR_INVALID_ARG;
  if (!aligned(xhat, 16) || !aligned(payload, 16) || !aligned(header, 4)) return ACCEPT_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->scheme == ACCEPT_UNIFORM)
    *launch_err = launch_uniform_decompress(*d, header, payload, xhat, s, tm);
  else
    *launch_err = launch_mbq_decompress(*d, header, payload, xhat, s, tm);
  return *launch_err == hipSuccess ? ACCEPT_OK : ACCEPT_ERR_HIP;
}

}  // namespace

extern "C" {

accept_status accept_packed_size(const accept_desc* desc, size_t* header_bytes, size_t* payload_bytes) {
  const accept_status st = check_desc(desc);
  if (st != ACCEPT_OK) return st;
  if (!header_bytes || !payload_bytes) return ACCEPT_ERR_INVALID_ARG;
  const int64_t k = desc->bits;
  if (desc->scheme == ACCEPT_MBQ) {
    *header_bytes = size_t(4 * (k + 1));
    *payload_bytes = desc->layout == ACCEPT_LAYOUT_UNENCODED ? size_t(desc->n * desc->m * k)
                                                             : size_t(((desc->n + 7) / 8) * desc->m * k);
  } else {
    const int64_t C = desc->channels > 1 ? desc->channels : 1;
    *header_bytes = size_t(4 * C);
    if (desc->layout == ACCEPT_LAYOUT_UNENCODED) {
      *payload_bytes = size_t(desc->n * desc->m);
    } else if (desc->layout == ACCEPT_LAYOUT_BATCH) {
      const int64_t per = 8 / k;
      *payload_bytes = size_t(((desc->n + per - 1) / per) * desc->m);
    } else {
      *payload_bytes = size_t((desc->n * desc->m * k + 7) / 8);
    }
  }
  return ACCEPT_OK;
}

accept_status accept_workspace_size(const accept_desc* desc, size_t* bytes) {
  const accept_status st = check_desc(desc);
  if (st != ACCEPT_OK) return st;
  if (!bytes) return ACCEPT_ERR_INVALID_ARG;
  *bytes = desc->scheme == ACCEPT_UNIFORM ? make_uplan(*desc).bytes : make_mplan(*desc).bytes;
  return ACCEPT_OK;
}

accept_status accept_compress(const accept_desc* desc, const void* x_dev, const float* alpha_prev_dev,
                              void* header_dev, void* payload_dev, void* workspace_dev, void* hip_stream) {
  hipError_t e;
  return do_compress(desc, x_dev, alpha_prev_dev, header_dev, payload_dev, workspace_dev, hip_stream, nullptr, &e);
}

accept_status accept_decompress(const accept_desc* desc, const void* header_dev, const void* payload_dev,
                                void* xhat_dev, void* hip_stream) {
  hipError_t e;
  return do_decompress(desc, header_dev, payload_dev, xhat_dev, hip_stream, nullptr, &e);
}

accept_status accept_compress_noalloc(const accept_desc* desc, const void* x_dev, const float* alpha_prev_dev,
                                      void* header_dev, void* payload_dev, void* hip_stream) {
  const accept_status st = check_desc(desc);
  if (st != ACCEPT_OK) return st;
  const size_t need = desc->scheme == ACCEPT_UNIFORM ? make_uplan(*desc).bytes : make_mplan(*desc).bytes;
  if (need > kScratchBytes) return ACCEPT_ERR_UNSUPPORTED;  // host-only check, before any HIP call
  void* ws = scratch_of_current_device();
  if (!ws) return ACCEPT_ERR_HIP;
  hipError_t e;
  return do_compress(desc, x_dev, alpha_prev_dev, header_dev, payload_dev, ws, hip_stream, nullptr, &e);
}

accept_status accept_mbq_init(const accept_desc* desc, const void* x_dev, float* alpha0_dev, void* workspace_dev,
                              void* hip_stream) {
  const accept_status st = check_desc(desc);
  if (st != ACCEPT_OK) return st;
  if (desc->scheme != ACCEPT_MBQ) return ACCEPT_ERR_INVALID_ARG;
  if (!x_dev || !alpha0_dev || !workspace_dev) return ACCEPT_ERR_INVALID_ARG;
  if (!aligned(x_dev, 16) || !aligned(alpha0_dev, 4) || !aligned(workspace_dev, 256)) return ACCEPT_ERR_INVALID_ARG;
  const MPlan p = make_mplan(*desc);
  const hipError_t e =
      launch_mbq_init(*desc, p, x_dev, alpha0_dev, nullptr, workspace_dev, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ACCEPT_OK : ACCEPT_ERR_HIP;
}

accept_status accept_mbq_compress_first(const accept_desc* desc, const void* x_dev, void* header_dev,
                                        void* payload_dev, void* workspace_dev, void* hip_stream) {
  const accept_status st = check_desc(desc);
  if (st != ACCEPT_OK) return st;
  if (desc->scheme != ACCEPT_MBQ || desc->layout != ACCEPT_LAYOUT_PACKED) return ACCEPT_ERR_INVALID_ARG;
  if (!x_dev || !header_dev || !payload_dev || !workspace_dev) return ACCEPT_ERR_INVALID_ARG;
  if (!aligned(x_dev, 16) || !aligned(payload_dev, 16) || !aligned(header_dev, 4) || !aligned(workspace_dev, 256))
    return ACCEPT_ERR_INVALID_ARG;
  const MPlan p = make_mplan(*desc);
  const hipError_t e = launch_mbq_init(*desc, p, x_dev, static_cast<float*>(header_dev), payload_dev, workspace_dev,
                                       static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ACCEPT_OK : ACCEPT_ERR_HIP;
}

accept_status accept_compress_timed(const accept_desc* desc, const void* x_dev, const float* alpha_prev_dev,
                                    void* header_dev, void* payload_dev, void* workspace_dev, void* hip_stream,
                                    float* stage_ms, int* n_stages) {
  if (!stage_ms || !n_stages) return ACCEPT_ERR_INVALID_ARG;
  *n_stages = 0;
  StageTimer tm;
  hipError_t e;
  const accept_status st =
      do_compress(desc, x_dev, alpha_prev_dev, header_dev, payload_dev, workspace_dev, hip_stream, &tm, &e);
  if (st != ACCEPT_OK && st != ACCEPT_ERR_HIP) return st;
  return finish_timer(tm, e, stage_ms, n_stages);
}

accept_status accept_decompress_timed(const accept_desc* desc, const void* header_dev, const void* payload_dev,
                                      void* xhat_dev, void* hip_stream, float* stage_ms, int* n_stages) {
  if (!stage_ms || !n_stages) return ACCEPT_ERR_INVALID_ARG;
  *n_stages = 0;
  StageTimer tm;
  hipError_t e;
  const accept_status st = do_decompress(desc, header_dev, payload_dev, xhat_dev, hip_stream, &tm, &e);
  if (st != ACCEPT_OK && st != ACCEPT_ERR_HIP) return st;
  return finish_timer(tm, e, stage_ms, n_stages);
}

const char* accept_stage_name(const accept_desc* desc, int is_decompress, int i) {
  if (check_desc(desc) != ACCEPT_OK || i < 0) return nullptr;
  const bool plain = desc->layout != ACCEPT_LAYOUT_PACKED;
  if (is_decompress) {
    if (i != 0) return nullptr;
    if (plain) return desc->scheme == ACCEPT_UNIFORM ? "dequant_plain" : "mbq_decode_plain";
    return desc->scheme == ACCEPT_UNIFORM ? "unpack_dequant" : "mbq_decode";
  }
  if (desc->scheme == ACCEPT_MBQ) {
    static const char* const names[] = {"mbq_encode", "mbq_finalize"};
    static const char* const names_plain[] = {"mbq_encode_plain", "mbq_finalize"};
    return i < 2 ? (plain ? names_plain[i] : names[i]) : nullptr;
  }
  if (plain) {
    static const char* const names[] = {"range", "range_finalize", "quantize_plain"};
    return i < 3 ? names[i] : nullptr;
  }
  if (desc->channels > 1 && !make_uplan(*desc).local_ranges) {
    static const char* const names[] = {"range", "range_finalize", "quantize_pack"};
    return i < 3 ? names[i] : nullptr;
  }
  static const char* const names[] = {"range", "quantize_pack"};
  return i < 2 ? names[i] : nullptr;
}

int accept_bits_schedule(int direction, int lr_changes_so_far) {
  if (lr_changes_so_far < 0) return -1;
  if (direction == 0) return lr_changes_so_far >= 2 ? 4 : 2 + lr_changes_so_far;
  if (direction == 1) return lr_changes_so_far == 0 ? 8 : 4;
  return -1;
}

const char* accept_status_string(accept_status status) {
  switch (status) {
    case ACCEPT_OK: return "ok";
    case ACCEPT_ERR_INVALID_ARG: return "invalid argument";
    case ACCEPT_ERR_UNSUPPORTED: return "unsupported";
    case ACCEPT_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case ACCEPT_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* accept_version(void) { return "0.1.0"; }

}  // extern "C"
