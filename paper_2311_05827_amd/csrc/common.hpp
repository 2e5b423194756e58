// Internal declarations shared by the HIP translation units of libaccept (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "accept.h"
#include "accept_profile.h"

namespace accept {

constexpr int kBlock = 256;       // threads per workgroup: 4 wavefronts of 64
constexpr int kWave = 64;
constexpr int kTileElems = 8192;  // elements one workgroup quantizes and packs per iteration

struct bf16_t {
  uint16_t bits;
};

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int VEC = 4;  // elements per 16-byte vector
};
template <>
struct Elem<bf16_t> {
  static constexpr int VEC = 8;
};

// ---- event bracketing for the *_timed entry points -------------------------------------
struct StageTimer {
  hipEvent_t ev[ACCEPT_MAX_STAGES + 1];
  int n = 0;
  bool failed = false;
  void mark(hipStream_t s) {
    if (n > ACCEPT_MAX_STAGES) return;
    if (hipEventCreate(&ev[n]) != hipSuccess) { failed = true; return; }
    if (hipEventRecord(ev[n], s) != hipSuccess) failed = true;
    ++n;
  }
};
inline void mark(StageTimer* t, hipStream_t s) {
  if (t) t->mark(s);
}

// Every workspace starts with a control block that the library keeps between calls: words that
// must be zero when a call starts and are put back to zero before it ends (the work counters of
// the multi-bit encoder).  The caller zero-fills the workspace once; no kernel of either scheme
// writes anything else there.
constexpr size_t kCtrlBytes = 16384;

// ---- scheme U (uniform) -----------------------------------------------------------------
enum UMode { U_TENSOR = 0, U_SEGMENTED = 1, U_GENERIC = 2 };

struct UPlan {
  int mode;
  int vec;             // elements per 16-byte vector of the input type
  int64_t N, m, C, seg_len;
  int range_grid;      // U_TENSOR: workgroups of the range kernel = number of partial maxima
  int64_t cps;         // U_SEGMENTED: chunks per segment
  int64_t chunk_vecs;  // U_SEGMENTED: 16-byte vectors per chunk
  int64_t items;       // U_SEGMENTED: n*C*cps partial maxima
  int col_tx;          // U_GENERIC: column threads per workgroup of the column pass (a power of two)
  int64_t col_grid_x;  // U_GENERIC: workgroups across the columns
  int col_grid_y;      // U_GENERIC: row blocks = maxima kept per column
  bool fast;           // vector path usable (every 16-byte vector lies inside one range group, or per_element)
  bool local_ranges;   // U_SEGMENTED: the quantize pass finishes the per-channel ranges itself, tile by tile
  bool per_element;    // U_GENERIC: one element per segment and rows of whole vectors (channels-last)
  size_t off_rtab;     // byte offset of the per-channel reciprocal table in the workspace
  size_t bytes;        // workspace bytes
};

UPlan make_uplan(const accept_desc& d);

hipError_t launch_uniform_compress(const accept_desc& d, const UPlan& p, const void* x, void* header,
                                   void* payload, void* ws, hipStream_t s, StageTimer* tm);
hipError_t launch_uniform_decompress(const accept_desc& d, const void* header, const void* payload,
                                     void* xhat, hipStream_t s, StageTimer* tm);

// ---- scheme M (multi-bit) ---------------------------------------------------------------
struct MPlan {
  int vec;                // columns per work item: 16-byte vectors when rows stay 16-byte aligned, else 1
  int64_t G;              // ceil(n/8) row groups
  int64_t items;          // G * (m / vec)
  bool stream;            // complete row groups go through the pipelined wave-item stream
  uint32_t wpg;           // wave-items (64 items) per row group
  uint32_t n_wave_items;  // of the complete row groups
  int grid;               // workgroups of the encode kernel = number of partial-sum records
  int nstat;              // doubles per record
  size_t bytes;
};

MPlan make_mplan(const accept_desc& d);

hipError_t launch_mbq_compress(const accept_desc& d, const MPlan& p, const void* x, const float* alpha_prev,
                               void* header, void* payload, void* ws, hipStream_t s, StageTimer* tm);
hipError_t launch_mbq_decompress(const accept_desc& d, const void* header, const void* payload, void* xhat,
                                 hipStream_t s, StageTimer* tm);
hipError_t launch_mbq_init(const accept_desc& d, const MPlan& p, const void* x, float* alpha_out, void* payload,
                           void* ws, hipStream_t s);

// ---- device helpers ---------------------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ float u32_as_f32(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f32_as_u32(float f) { return __float_as_uint(f); }

typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));

// Cache policy.  Tensors here are far larger than the caches and each byte is used once per
// kernel.  Streaming (non-temporal) stores let output lines drain to HBM while the kernel that
// wrote them still runs, instead of sitting dirty in L2 / the memory-side cache and stealing
// bandwidth from the next kernel; streaming loads keep single-use input from evicting them.
__device__ __forceinline__ uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  const v4u_t v = __builtin_nontemporal_load(reinterpret_cast<const v4u_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16_stream(void* p, uint4 v) {
  const v4u_t u = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(u, reinterpret_cast<v4u_t*>(p));
}

// NDW consecutive dwords of payload (plain stores: streaming stores of the payload gained nothing),
// aligned to 16 bytes when NDW % 4 == 0, to 8 when NDW % 2 == 0, else 4.
template <int NDW>
__device__ __forceinline__ void store_dwords(uint32_t* p, const uint32_t (&v)[NDW]) {
  struct alignas((NDW % 4 == 0) ? 16 : (NDW % 2 == 0) ? 8 : 4) Block { uint32_t w[NDW]; };
  Block b;
#pragma unroll
  for (int i = 0; i < NDW; ++i) b.w[i] = v[i];
  *reinterpret_cast<Block*>(p) = b;
}

// The same with streaming stores (the MBQ encoder's planes: fewer dirty lines are left for the
// end of the kernel, which the finalize kernel's start waits for).
template <int NDW>
__device__ __forceinline__ void store_dwords_stream(uint32_t* p, const uint32_t (&v)[NDW]) {
  if constexpr (NDW % 4 == 0) {
#pragma unroll
    for (int i = 0; i < NDW; i += 4) {
      const v4u_t u = {v[i], v[i + 1], v[i + 2], v[i + 3]};
      __builtin_nontemporal_store(u, reinterpret_cast<v4u_t*>(p + i));
    }
  } else if constexpr (NDW % 2 == 0) {
    typedef uint32_t v2u_t __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int i = 0; i < NDW; i += 2) {
      const v2u_t u = {v[i], v[i + 1]};
      __builtin_nontemporal_store(u, reinterpret_cast<v2u_t*>(p + i));
    }
  } else {
#pragma unroll
    for (int i = 0; i < NDW; ++i) __builtin_nontemporal_store(v[i], p + i);
  }
}

__device__ __forceinline__ void widen(const uint4 v, float (&f)[4]) {
  f[0] = u32_as_f32(v.x); f[1] = u32_as_f32(v.y); f[2] = u32_as_f32(v.z); f[3] = u32_as_f32(v.w);
}
__device__ __forceinline__ void widen(const uint4 v, float (&f)[8]) {  // eight bfloat16, element 0 in the low half
  f[0] = u32_as_f32(v.x << 16); f[1] = u32_as_f32(v.x & 0xFFFF0000u);
  f[2] = u32_as_f32(v.y << 16); f[3] = u32_as_f32(v.y & 0xFFFF0000u);
  f[4] = u32_as_f32(v.z << 16); f[5] = u32_as_f32(v.z & 0xFFFF0000u);
  f[6] = u32_as_f32(v.w << 16); f[7] = u32_as_f32(v.w & 0xFFFF0000u);
}
// 16-byte vector load widened to float32; the _stream form is for data read once.
__device__ __forceinline__ void load_vec(const float* p, float (&f)[4]) { widen(load16(p), f); }
__device__ __forceinline__ void load_vec(const bf16_t* p, float (&f)[8]) { widen(load16(p), f); }
__device__ __forceinline__ void load_vec_stream(const float* p, float (&f)[4]) { widen(load16_stream(p), f); }
__device__ __forceinline__ void load_vec_stream(const bf16_t* p, float (&f)[8]) { widen(load16_stream(p), f); }
__device__ __forceinline__ float load_one(const float* p) { return *p; }
__device__ __forceinline__ float load_one(const bf16_t* p) { return u32_as_f32(uint32_t(p->bits) << 16); }

// float32 -> bfloat16 bits, round to nearest even (finite values).
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t b = f32_as_u32(f);
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}
// 16-byte vector store of decompressed values (streaming).
__device__ __forceinline__ void store_vec(float* p, const float (&f)[4]) {
  store16_stream(p, make_uint4(f32_as_u32(f[0]), f32_as_u32(f[1]), f32_as_u32(f[2]), f32_as_u32(f[3])));
}
__device__ __forceinline__ void store_vec(bf16_t* p, const float (&f)[8]) {
  uint4 v;
  v.x = bf16_rne(f[0]) | (bf16_rne(f[1]) << 16);
  v.y = bf16_rne(f[2]) | (bf16_rne(f[3]) << 16);
  v.z = bf16_rne(f[4]) | (bf16_rne(f[5]) << 16);
  v.w = bf16_rne(f[6]) | (bf16_rne(f[7]) << 16);
  store16_stream(p, v);
}
__device__ __forceinline__ void store_one(float* p, float f) { *p = f; }
__device__ __forceinline__ void store_one(bf16_t* p, float f) { p->bits = uint16_t(bf16_rne(f)); }

// Four consecutive elements (16 bytes of float32, 8 bytes of bfloat16; p aligned to that).
template <typename T>
__device__ __forceinline__ void load_quad(const T* p, float (&f)[4]) {
  if constexpr (sizeof(T) == 4) {
    widen(load16_stream(p), f);
  } else {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    f[0] = u32_as_f32(v.x << 16); f[1] = u32_as_f32(v.x & 0xFFFF0000u);
    f[2] = u32_as_f32(v.y << 16); f[3] = u32_as_f32(v.y & 0xFFFF0000u);
  }
}
template <typename T>
__device__ __forceinline__ void store_quad(T* p, const float (&f)[4]) {
  if constexpr (sizeof(T) == 4) {
    store_vec(p, f);
  } else {
    uint2 v;
    v.x = bf16_rne(f[0]) | (bf16_rne(f[1]) << 16);
    v.y = bf16_rne(f[2]) | (bf16_rne(f[3]) << 16);
    *reinterpret_cast<uint2*>(p) = v;
  }
}

// Lane exchange inside a row of 16 lanes with a DPP control word (all lanes stay valid).
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return uint32_t(__builtin_amdgcn_update_dpp(int(v), int(v), CTRL, 0xF, 0xF, false));
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// Maximum over the 64 lanes of a wavefront; every lane receives the result.  Operands are
// non-negative floats, compared through their bit patterns' float view.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, u32_as_f32(dpp_u32<kDppQuadSwap1>(f32_as_u32(v))));
  v = fmaxf(v, u32_as_f32(dpp_u32<kDppQuadSwap2>(f32_as_u32(v))));
  v = fmaxf(v, u32_as_f32(dpp_u32<kDppRowHalfMirror>(f32_as_u32(v))));
  v = fmaxf(v, u32_as_f32(dpp_u32<kDppRowMirror>(f32_as_u32(v))));
  v = fmaxf(v, __shfl_xor(v, 16, kWave));
  v = fmaxf(v, __shfl_xor(v, 32, kWave));
  return v;
}

// Lane exchange of a float64 inside a row of 16 lanes (two 32-bit DPP moves).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const uint64_t b = uint64_t(__double_as_longlong(v));
  const uint32_t lo = dpp_u32<CTRL>(uint32_t(b)), hi = dpp_u32<CTRL>(uint32_t(b >> 32));
  return __longlong_as_double((long long)((uint64_t(hi) << 32) | lo));
}
__device__ __forceinline__ double readlane_f64(double v, int lane) {
  const uint64_t b = uint64_t(__double_as_longlong(v));
  const uint32_t lo = uint32_t(__builtin_amdgcn_readlane(int(uint32_t(b)), lane));
  const uint32_t hi = uint32_t(__builtin_amdgcn_readlane(int(uint32_t(b >> 32)), lane));
  return __longlong_as_double((long long)((uint64_t(hi) << 32) | lo));
}

// Sum over the 64 lanes in a fixed order (so the result does not depend on timing); every lane
// receives the same value.  Four butterfly steps inside each row of 16 lanes (partners add in
// either order: the same float64 either way), then the four row sums as (r0 + r1) + (r2 + r3).
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_f64<kDppQuadSwap1>(v);
  v += dpp_f64<kDppQuadSwap2>(v);
  v += dpp_f64<kDppRowHalfMirror>(v);
  v += dpp_f64<kDppRowMirror>(v);
  const double r0 = readlane_f64(v, 0), r1 = readlane_f64(v, 16), r2 = readlane_f64(v, 32), r3 = readlane_f64(v, 48);
  return (r0 + r1) + (r2 + r3);
}

// Loads and stores that are coherent across the whole device although every group of compute
// units has a second-level cache of its own: they go through to memory instead of staying in
// (or being served from) that cache.  For the few words workgroups hand to each other inside
// one kernel.
__device__ __forceinline__ void store_device_scope(double* p, double v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double load_device_scope(const double* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// u in [0,1) on a 2^-24 grid: top 24 bits of splitmix64's output function at
// seed + (idx+1) * 0x9E3779B97F4A7C15.
__device__ __forceinline__ float counter_uniform(uint64_t seed, uint64_t idx) {
  uint64_t z = seed + (idx + 1ull) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  return float(uint32_t(z >> 40)) * 0x1p-24f;
}

#endif  // __HIPCC__

}  // namespace accept
