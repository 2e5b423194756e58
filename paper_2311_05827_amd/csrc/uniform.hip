// Scheme U on gfx950: max-abs range reduction, fused quantize + dense bit pack, fused
// unpack + dequantize (paper paragraphs "Backward Quantizer", "Backward Encoder",
// "Backward Decoder", "Backward Dequantizer"; generalised from k in {4, 8} to k in 2..8
// and to per-channel ranges).
//
// Data movement design: all tensor traffic is 16-byte vector loads/stores that are
// contiguous across the 64 lanes of a wavefront.  The only cross-lane exchange in the
// compressor is one LDS round trip of already-quantized 4-code "pieces" (4k bits each):
// 8 pieces = 32 codes = exactly k dwords for every k, so one lane can emit whole dwords and
// no global atomics are needed even when codes straddle dword boundaries.
#include "common.hpp"

namespace accept {

namespace {

// The range pass reads the end of the tensor with ordinary (cacheable) loads: the quantize pass
// reads the same tensor again right after it, last-read data first, and finds that part still
// in the memory-side cache (streaming loads would leave nothing there).  What lies more than
// kRangeKeepBytes before the end is read with streaming loads: little of it would survive until
// the quantize pass gets there, cacheable loads are the slower kind, most of all behind a kernel
// whose stores are still draining, and whatever they bring into the memory-side cache pushes
// out what other kernels left there (the payload a decoder is about to read, for one).
constexpr int64_t kRangeKeepBytes = int64_t(64) << 20;  // a quarter of the 256 MiB memory-side cache
template <typename T, int V>
__device__ __forceinline__ void load_range(const T* p, float (&f)[V]) {
  widen(load16(p), f);
}

constexpr float kTinyRange = 0x1p-100f;     // smaller ranges count as an all-zero tensor
constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23: adding it rounds to integer, half to even
constexpr int kRangeGridMax = 512;     // partial maxima of the per-tensor range pass
constexpr int kQuantGridMax = 2048;    // workgroups of the quantize+pack kernel
constexpr int kDequantGridMax = 8192;
static_assert(kQuantGridMax % 8 == 0 && kRangeGridMax % 8 == 0, "grids at their caps keep tile and workgroup index equal modulo 8");
static_assert(kRangeGridMax <= 4096, "the workspace holds at most 4096 partial maxima");

// s = c / L and r = L / c as correctly rounded float32 quotients (L is a small integer, exact in
// float32; __fdiv_rn is the IEEE round-to-nearest-even division).
__device__ __forceinline__ void scale_from_range(float c, int k, float& s, float& r) {
  const float L = float((1 << (k - 1)) - 1);
  if (c >= kTinyRange) {
    s = __fdiv_rn(c, L);
    r = __fdiv_rn(L, c);
  } else {
    s = 0.0f;
    r = 0.0f;
  }
}

// Position of a 16-byte vector inside the channel structure, advanced without divisions.
struct ChanPos {
  int64_t rem;  // vector offset inside the current segment, < seg_vecs
  int32_t ch;   // channel of the current segment, < C
};
struct ChanStep {
  int64_t dr;   // step mod seg_vecs
  int32_t dch;  // (step / seg_vecs) mod C
};
struct ChanGeom {
  int64_t seg_vecs;  // vectors per segment (segment = one channel of one batch row)
  int32_t C;
  ChanStep s256;     // step of 256 vectors
  ChanStep sgrid;    // step of one grid stride (gridDim.x tiles, or gridDim.x*256 vectors)
};
__device__ __forceinline__ ChanPos chan_init(const ChanGeom& g, int64_t vec_index) {
  ChanPos p;
  const int64_t seg = vec_index / g.seg_vecs;
  p.rem = vec_index - seg * g.seg_vecs;
  p.ch = int32_t(seg % g.C);
  return p;
}
__device__ __forceinline__ void chan_advance(const ChanGeom& g, ChanPos& p, const ChanStep& st) {
  p.rem += st.dr;
  int32_t carry = 0;
  if (p.rem >= g.seg_vecs) { p.rem -= g.seg_vecs; carry = 1; }
  p.ch += st.dch + carry;
  if (p.ch >= g.C) p.ch -= g.C;
}

// kRangePerVectorLocal: the range pass left `per` partial maxima for every channel, those of
// channel ch at partials[ch * per ..].
struct LocalRanges {
  int32_t per;
};
// Used for segments of at least 2048 elements; a tile is 8192 elements: it touches at most
// 8192/2048 + 1 segments.
constexpr int kLocalRanges = 8;
constexpr int kLocalMinSegment = 2048;
static_assert(kTileElems / kLocalMinSegment + 1 <= kLocalRanges, "entries of a tile's table");
__device__ __forceinline__ void chan_retreat(const ChanGeom& g, ChanPos& p, const ChanStep& st) {
  p.rem -= st.dr;
  int32_t borrow = 0;
  if (p.rem < 0) { p.rem += g.seg_vecs; borrow = 1; }
  p.ch -= st.dch + borrow;
  if (p.ch < 0) p.ch += g.C;
}

// How the elements of a 16-byte vector find their range group (the fast paths of the quantizer
// and of the decoder are compiled once per case):
constexpr int kOneRange = 0;         // one group for the tensor
constexpr int kRangePerVector = 1;   // segments are whole vectors: one group per vector, ChanPos.ch its channel
constexpr int kRangePerElement = 2;  // one element per segment (channels-last) and rows of whole vectors:
                                     // ChanPos.ch is the vector's place in its row, element e has channel ch*VEC + e
constexpr int kRangePerVectorLocal = 3;  // as kRangePerVector, quantizer only: no table in memory yet, the workgroup
                                         // finishes the ranges of each tile's channels itself; ChanPos.ch then indexes
                                         // its own small table (channel minus the tile's first channel, modulo C)
// The per-group values (reciprocals for the quantizer, scales for the decoder) of a vector's elements.
template <int MODE, int VEC>
__device__ __forceinline__ void ranges_of_vector(const float* __restrict__ tab, float one, int32_t ch,
                                                 float (&out)[VEC]) {
  if constexpr (MODE == kRangePerElement) {
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) {
      const float4 t = *reinterpret_cast<const float4*>(tab + int64_t(ch) * VEC + 4 * h);  // tab is 16-byte aligned
      out[4 * h] = t.x; out[4 * h + 1] = t.y; out[4 * h + 2] = t.z; out[4 * h + 3] = t.w;
    }
  } else {
    const float v = MODE == kOneRange ? one : tab[ch];
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = v;
  }
}

// =========================================================================== range (U1)
// One range for the tensor: workgroup b reads the tiles b, b + grid, ... (the quantize pass's
// tiles, 8192 consecutive elements, all of a thread's 16-byte loads of a tile in flight together),
// DPP wave reduction, one partial maximum per workgroup.  max is exact and order independent, so
// the result is reproducible without atomics or a fixed order.  Tile t is read by a workgroup whose
// index is t modulo 8 (grids of more than 8 workgroups are multiples of 8): under round-robin
// dispatch that is also the die whose L2 the quantize pass reads tile t through.
template <typename T>
__global__ __launch_bounds__(kBlock) void range_tensor_kernel(const T* __restrict__ x, int64_t N,
                                                               float* __restrict__ partials) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int LOADS = kTileElems / (kBlock * VEC);  // vectors per thread per tile
  __shared__ float red[kBlock / kWave];
  const int64_t nvec = N / VEC;
  const int64_t full_tiles = N / kTileElems;
  float c = 0.0f;
  constexpr int64_t KEEP_TILES = kRangeKeepBytes / int64_t(kTileElems * sizeof(T));
  const int64_t stream_tiles = full_tiles > KEEP_TILES ? full_tiles - KEEP_TILES : 0;
  int64_t tile = blockIdx.x;
  for (; tile < stream_tiles; tile += gridDim.x) {  // streaming loads
    const T* xt = x + tile * kTileElems;
    float f[LOADS][VEC];
#pragma unroll
    for (int u = 0; u < LOADS; ++u) load_vec_stream(xt + (u * kBlock + threadIdx.x) * VEC, f[u]);
#pragma unroll
    for (int u = 0; u < LOADS; ++u)
#pragma unroll
      for (int e = 0; e < VEC; ++e) c = fmaxf(c, fabsf(f[u][e]));
  }
  for (; tile < full_tiles; tile += gridDim.x) {  // cacheable loads
    const T* xt = x + tile * kTileElems;
    float f[LOADS][VEC];
#pragma unroll
    for (int u = 0; u < LOADS; ++u) load_range<T, VEC>(xt + (u * kBlock + threadIdx.x) * VEC, f[u]);
#pragma unroll
    for (int u = 0; u < LOADS; ++u)
#pragma unroll
      for (int e = 0; e < VEC; ++e) c = fmaxf(c, fabsf(f[u][e]));
  }
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  for (int64_t v = full_tiles * (kTileElems / VEC) + int64_t(blockIdx.x) * kBlock + threadIdx.x; v < nvec;
       v += stride) {
    float f[VEC];
    load_range<T, VEC>(x + v * VEC, f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) c = fmaxf(c, fabsf(f[e]));
  }
  if (blockIdx.x == 0 && int64_t(threadIdx.x) < N - nvec * VEC)
    c = fmaxf(c, fabsf(load_one(x + nvec * VEC + threadIdx.x)));
  c = wave_max(c);
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    float b = red[0];
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) b = fmaxf(b, red[w]);
    partials[blockIdx.x] = b;
  }
}

// One range per channel, long segments: one wavefront reduces one chunk of one segment
// (segment = channel ch of batch row r, contiguous in memory; chunks are at most a tile long);
// partial index = (ch*cps + chunk)*rows + r: the maxima of one channel lie together.  Workgroup t takes the chunks that begin inside tile t
// of the quantize pass (8192 consecutive elements), its wavefronts in turn: the data a die reads
// here is, up to a chunk's overhang, the data the quantize pass reads through the same die's L2.
template <typename T>
__global__ __launch_bounds__(kBlock) void range_segments_kernel(const T* __restrict__ x, int64_t items, int64_t cps,
                                                                 int64_t seg_vecs, int64_t chunk_vecs, int64_t rows,
                                                                 int64_t C, float* __restrict__ partials) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int64_t TILE_VECS = kTileElems / VEC;
  const int lane = threadIdx.x & (kWave - 1);
  // first chunk that begins at or after vector a: the segment of a, and the chunk of a rounded up
  auto first_item_from = [&](int64_t a) {
    int64_t sid = a / seg_vecs;
    int64_t chunk = (a - sid * seg_vecs + chunk_vecs - 1) / chunk_vecs;
    if (chunk >= cps) { sid += 1; chunk = 0; }
    const int64_t it = sid * cps + chunk;
    return it < items ? it : items;
  };
  const int64_t it_lo = first_item_from(int64_t(blockIdx.x) * TILE_VECS);
  const int64_t it_hi = blockIdx.x + 1 == gridDim.x ? items : first_item_from((int64_t(blockIdx.x) + 1) * TILE_VECS);
  for (int64_t it = it_lo + threadIdx.x / kWave; it < it_hi; it += kBlock / kWave) {
    const int64_t sid = it / cps;
    const int64_t chunk = it - sid * cps;
    const int64_t first = chunk * chunk_vecs;
    int64_t count = seg_vecs - first;
    if (count > chunk_vecs) count = chunk_vecs;
    const T* base = x + (sid * seg_vecs + first) * VEC;
    float c = 0.0f;
    // eight loads in flight per lane, kept as raw vectors until used; a lane whose turn lies
    // beyond the chunk's end re-reads the chunk's last vector (a maximum does not mind), so that
    // the loads stay unconditional and a chunk's last vectors do not cost a trip to memory each
    // (a chunk that begins in the part of the tensor that is read with streaming loads: see
    // kRangeKeepBytes; the choice is the same for all lanes of the wavefront)
    const bool stream = (sid * seg_vecs + first) * int64_t(VEC * sizeof(T)) + kRangeKeepBytes <
                        items / cps * seg_vecs * int64_t(VEC * sizeof(T));
    for (int64_t j = lane; j < count; j += 8 * kWave) {
      uint4 raw[8];
      if (stream) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          int64_t idx = j + u * kWave;
          if (idx >= count) idx = count - 1;
          raw[u] = load16_stream(base + idx * VEC);
        }
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          int64_t idx = j + u * kWave;
          if (idx >= count) idx = count - 1;
          raw[u] = load16(base + idx * VEC);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float f[VEC];
        widen(raw[u], f);
#pragma unroll
        for (int e = 0; e < VEC; ++e) c = fmaxf(c, fabsf(f[e]));
      }
    }
    c = wave_max(c);  // every lane of the wavefront reaches this point: the loop bounds are wave-uniform
    const int64_t row = sid / C;
    if (lane == 0) partials[((sid - row * C) * cps + chunk) * rows + row] = c;
  }
}

// One range per channel, any other geometry (short segments, segments that no 16-byte vector
// respects; with one element per segment this is a channels-last tensor): two stages, no atomics.
// Stage 1 works on columns: a thread owns CV adjacent columns (a 16-byte vector when rows keep
// vectors aligned, else one column), walks down its share of the rows and keeps the columns'
// maxima; the workgroup is TX column-threads wide (consecutive lanes read consecutive vectors of
// a row) and 256/TX rows high; its threads of equal column meet in local memory and the
// workgroup writes one maximum per column: colmax[by * m + column].  Stage 2 folds the columns
// of a channel and the row blocks.
template <typename T, int CV>
__global__ __launch_bounds__(kBlock) void range_columns_kernel(const T* __restrict__ x, int64_t n, int64_t m,
                                                                int tx_threads, float* __restrict__ colmax) {
  __shared__ float red[kBlock][CV];
  const int ty_threads = kBlock / tx_threads;
  const int tx = threadIdx.x % tx_threads, ty = threadIdx.x / tx_threads;
  const int64_t ncv = m / CV;
  const int64_t cv = int64_t(blockIdx.x) * tx_threads + tx;
  float c[CV];
#pragma unroll
  for (int e = 0; e < CV; ++e) c[e] = 0.0f;
  if (cv < ncv) {
    const int64_t row_step = int64_t(gridDim.y) * ty_threads;
    int64_t r = int64_t(blockIdx.y) * ty_threads + ty;
    const T* col = x + cv * CV;
    for (; r + 3 * row_step < n; r += 4 * row_step) {  // four loads in flight
      float f[4][CV];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if constexpr (CV > 1) load_range<T, CV>(col + (r + u * row_step) * m, f[u]);
        else f[u][0] = load_one(col + (r + u * row_step) * m);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < CV; ++e) c[e] = fmaxf(c[e], fabsf(f[u][e]));
    }
    for (; r < n; r += row_step) {
      float f[CV];
      if constexpr (CV > 1) load_range<T, CV>(col + r * m, f);
      else f[0] = load_one(col + r * m);
#pragma unroll
      for (int e = 0; e < CV; ++e) c[e] = fmaxf(c[e], fabsf(f[e]));
    }
  }
#pragma unroll
  for (int e = 0; e < CV; ++e) red[threadIdx.x][e] = c[e];
  __syncthreads();
  if (ty == 0 && cv < ncv) {
    for (int y = 1; y < ty_threads; ++y)
#pragma unroll
      for (int e = 0; e < CV; ++e) c[e] = fmaxf(c[e], red[y * tx_threads + tx][e]);
#pragma unroll
    for (int e = 0; e < CV; ++e) colmax[int64_t(blockIdx.y) * m + cv * CV + e] = c[e];
  }
}

// Stage 2 and U1b: one workgroup per channel takes the maximum over the channel's seg_len
// columns in all nby row blocks, writes s to the header and the reciprocal to the table.
// Thread t starts at entry t of the channel's seg_len x nby maxima (row block t / seg_len,
// column t % seg_len) and steps by 256 entries, carried as (row block, column) so that the
// loop needs no division.
__global__ __launch_bounds__(kBlock) void range_columns_finalize_kernel(const float* __restrict__ colmax, int64_t m,
                                                                        int64_t seg_len, int nby, int k,
                                                                        float* __restrict__ header,
                                                                        float* __restrict__ rtab) {
  __shared__ float red[kBlock / kWave];
  const int64_t ch = blockIdx.x;
  const float* base = colmax + ch * seg_len;
  const int64_t dby = int64_t(kBlock) / seg_len, dq = int64_t(kBlock) % seg_len;
  int64_t by = int64_t(threadIdx.x) / seg_len, q = int64_t(threadIdx.x) % seg_len;
  float c = 0.0f;
  while (by < nby) {
    float v[4];  // four loads in flight
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      v[u] = by < nby ? base[by * m + q] : 0.0f;
      by += dby;
      q += dq;
      if (q >= seg_len) { q -= seg_len; ++by; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) c = fmaxf(c, v[u]);
  }
  c = wave_max(c);
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) c = fmaxf(c, red[w]);
    float s, r;
    scale_from_range(c, k, s, r);
    header[ch] = s;
    rtab[ch] = r;
  }
}

// U1b per channel: reduce the channel's `per` partial maxima (they lie together, channel after
// channel), write s to the header and the reciprocal r to the workspace table.  One wavefront
// per channel.
__global__ __launch_bounds__(kWave) void range_finalize_kernel(const float* __restrict__ partials, int64_t per, int k,
                                                                float* __restrict__ header, float* __restrict__ rtab) {
  const int64_t ch = blockIdx.x;
  float c = 0.0f;
  for (int64_t j = threadIdx.x; j < per; j += kWave) c = fmaxf(c, partials[ch * per + j]);
  c = wave_max(c);
  if (threadIdx.x == 0) {
    float s, r;
    scale_from_range(c, k, s, r);
    header[ch] = s;
    rtab[ch] = r;
  }
}

// =========================================================================== quantize (U2)
// One element: v = x * r (one float32 multiply), round, clamp, offset to a k-bit code.
template <int K, bool STOCH>
__device__ __forceinline__ uint32_t quantize1(float f, float r, uint64_t seed, int64_t idx) {
  constexpr int HALF = 1 << (K - 1);
  constexpr uint32_t MASK = (1u << K) - 1u;
  const float v = __fmul_rn(f, r);
  if (!STOCH) {
    // Round half to even through the magic-number add.  |v| <= L(1 + 2^-23), so the rounded
    // value lies in [-L, L] and the clamp of the definition never binds; the mask only keeps
    // codes of non-finite inputs inside their k bits.  The sum's low mantissa bits are
    // q + HALF (k < 8) or q mod 256 (k = 8).
    const float t = __fadd_rn(v, kRoundMagic + float(K == 8 ? 0 : HALF));
    return f32_as_u32(t) & MASK;
  }
  const float fl = floorf(v);
  const float pr = __fsub_rn(v, fl);  // exact
  const float u = counter_uniform(seed, uint64_t(idx));
  int q = int(fl) + (u < pr ? 1 : 0);
  q = min(max(q, -HALF), HALF - 1);
  return (K == 8) ? (uint32_t(q) & 0xFFu) : uint32_t(q + HALF);
}

// Four consecutive elements -> one 4k-bit piece, first element most significant.
template <int K, bool STOCH>
__device__ __forceinline__ uint32_t quantize4(const float* f, const float* r, uint64_t seed, int64_t idx0) {
  uint32_t piece = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) piece = (piece << K) | quantize1<K, STOCH>(f[e], r[e], seed, idx0 + e);
  return piece;
}

// U3 for 32 consecutive codes: eight 4k-bit pieces -> k dwords of the big-endian bit
// stream, each dword byte-swapped into memory order.
template <int K>
__device__ __forceinline__ void pack8(const uint32_t (&P)[8], uint32_t (&out)[K]) {
  constexpr int W = 4 * K;
  uint64_t acc = 0;
  int nb = 0, o = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    acc = (W == 32) ? ((acc << 32) | P[i]) : ((acc << W) | P[i]);
    nb += W;
    if (nb >= 32) {
      out[o++] = __builtin_bswap32(uint32_t(acc >> (nb - 32)));
      nb -= 32;
    }
  }
}

// Slow path for one group of 8 elements -> k bytes (tails and odd channel geometries):
// scalar loads, per-byte stores guarded by the payload size.  Elements at or beyond N
// contribute zero bits.
template <typename T, int K, bool STOCH, typename RFn>
__device__ __forceinline__ void quantize_group8(const T* __restrict__ x, uint8_t* __restrict__ payload, int64_t grp,
                                                int64_t N, int64_t payload_bytes, uint64_t seed, RFn r_of) {
  uint64_t acc = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int64_t i = grp * 8 + e;
    uint64_t code = 0;
    if (i < N) code = quantize1<K, STOCH>(load_one(x + i), r_of(i), seed, i);
    acc = (acc << K) | code;
  }
#pragma unroll
  for (int b = 0; b < K; ++b) {
    const int64_t byte = grp * K + b;
    if (byte < payload_bytes) payload[byte] = uint8_t(acc >> (8 * (K - 1 - b)));
  }
}

// Fused U2 + U3.  Per iteration a workgroup takes one tile of 8192 consecutive elements:
// every thread loads 16-byte vectors (contiguous across lanes), quantizes them into pieces,
// parks the pieces in LDS; after one barrier thread g reads pieces 8g..8g+7 (32 consecutive
// elements) and emits k contiguous dwords.  The piece buffer is double buffered so that one
// barrier per tile is enough.  MODE says where an element's range comes from (kOneRange ..
// kRangePerVectorLocal above).  kOneRange folds U1b into the prologue: every workgroup reduces
// the range pass's partial maxima itself and workgroup 0 writes s to the header;
// kRangePerVectorLocal folds it into the tile loop (see local_r below); the other two modes read
// the table that a U1b kernel has written.  Elements after the last whole tile take the slow
// path at the end.
template <typename T, int K, int MODE, bool STOCH>
__global__ __launch_bounds__(kBlock) void quantize_pack_kernel(
    const T* __restrict__ x, uint32_t* __restrict__ payload32, float* __restrict__ header,
    const float* __restrict__ partials, int npart, const float* __restrict__ rtab, int64_t N, int64_t full_tiles,
    int64_t rev_tiles, int64_t slow_first_group, int64_t payload_bytes, ChanGeom geom, LocalRanges local, int64_t m,
    int64_t seg_len, uint64_t seed) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int64_t TILE_VECS = kTileElems / VEC;
  constexpr int QPV = VEC / 4;                       // pieces per vector
  constexpr int LOADS = kTileElems / (kBlock * VEC);  // vectors per thread per tile
  constexpr int PIECES = kTileElems / 4;
  __shared__ __attribute__((aligned(16))) uint32_t pieces[2][PIECES];
  __shared__ float red[kBlock / kWave];

  const int tid = threadIdx.x;
  // Tile order.  The range pass has just read the tensor front to back, so its end is what the
  // caches still hold: the first rev_tiles tiles (a multiple of 8, as is the grid then) are taken
  // last to first in groups of eight, tile = rev_tiles - 8 - 8*(i / 8) + i % 8 for the i-th tile
  // of the plain order.  A workgroup's tiles then step backwards by one grid stride, and tile and
  // workgroup index stay equal modulo 8: the die that read a tile in the range pass reads it
  // again here.  The up to seven tiles after rev_tiles keep their plain places.
  auto tile_of = [&](int64_t tile_f) {
    return tile_f < rev_tiles ? rev_tiles - 8 - (tile_f & ~int64_t(7)) + (tile_f & 7) : tile_f;
  };
  // A tile's vectors are asked for one tile ahead: those of the first tile here, before anything
  // else, those of every later tile as soon as the tile before it has been quantized.
  uint4 raw[LOADS];
  auto ask_for_tile = [&](int64_t tile) {
    const T* xt = x + tile * kTileElems;
#pragma unroll
    for (int u = 0; u < LOADS; ++u) raw[u] = load16_stream(xt + (u * kBlock + tid) * VEC);
  };
  if (int64_t(blockIdx.x) < full_tiles) ask_for_tile(tile_of(blockIdx.x));

  float r_tensor = 0.0f;
  if (MODE == kOneRange) {
    float c = 0.0f;
    for (int i = tid; i < npart; i += kBlock) c = fmaxf(c, partials[i]);
    c = wave_max(c);
    if ((tid & (kWave - 1)) == 0) red[tid / kWave] = c;
    __syncthreads();
    c = red[0];
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) c = fmaxf(c, red[w]);
    float s;
    scale_from_range(c, K, s, r_tensor);
    if (blockIdx.x == 0 && tid == 0) header[0] = s;
  }

  // Channel position of a tile's first vector (the same in all threads), stepped from tile to
  // tile; a thread's own position is that plus its index.
  ChanPos first_pos{0, 0};
  ChanStep mine{0, 0};
  if (MODE != kOneRange && int64_t(blockIdx.x) < full_tiles) {
    first_pos = chan_init(geom, tile_of(blockIdx.x) * TILE_VECS);
    mine.dr = int64_t(tid) % geom.seg_vecs;
    mine.dch = int32_t((int64_t(tid) / geom.seg_vecs) % geom.C);
  }

  // kRangePerVectorLocal: the reciprocals of the channels a tile touches, entry t for channel
  // (first channel of the tile + t) mod C, t < min(segments the tile touches, C).  Wavefront w
  // fills the entries w, w+4, ...: the maximum over the channel's `per` partial maxima (at most
  // two per lane), then U1b; the workgroup whose tile holds the start of the channel's segment
  // of batch row 0 writes s to the header.  A table is filled one tile ahead (it is double
  // buffered like the pieces, and the tile's one barrier publishes it): the partial maxima are
  // asked for before the tile is quantized and looked at after, so that their way from memory
  // (another die wrote them) is not waited for.
  constexpr int kLocalPerLane = 2, kLocalPerWave = kLocalRanges / (kBlock / kWave);
  static_assert(kLocalRanges % (kBlock / kWave) == 0, "entries per wavefront");
  __shared__ float local_r[2][kLocalRanges];
  struct LocalFetch {
    float v[kLocalPerWave][kLocalPerLane];
  };
  const int lane = tid & (kWave - 1);
  // does entry t exist for a tile whose first vector sits `rem` vectors into its segment?
  auto local_entry = [&](int t, const ChanPos& p0) {
    return t < geom.C && int64_t(t) * geom.seg_vecs - p0.rem < TILE_VECS;
  };
  auto local_fetch = [&](const ChanPos& p0, LocalFetch& lf) {
#pragma unroll
    for (int e = 0; e < kLocalPerWave; ++e) {
      const int t = tid / kWave + e * (kBlock / kWave);
      int32_t ch = p0.ch + t;
      if (ch >= geom.C) ch -= geom.C;
      const bool has = local_entry(t, p0);
#pragma unroll
      for (int l = 0; l < kLocalPerLane; ++l) {
        const int i = lane + l * kWave;
        lf.v[e][l] = (has && i < local.per) ? partials[uint32_t(ch * local.per + i)] : 0.0f;  // C * per < 2^31 (host)
      }
    }
  };
  auto local_finish = [&](int64_t tile, const ChanPos& p0, const LocalFetch& lf, float* table) {
#pragma unroll
    for (int e = 0; e < kLocalPerWave; ++e) {
      const int t = tid / kWave + e * (kBlock / kWave);
      if (!local_entry(t, p0)) break;  // the same in all lanes of the wavefront
      float c = lf.v[e][0];
#pragma unroll
      for (int l = 1; l < kLocalPerLane; ++l) c = fmaxf(c, lf.v[e][l]);
      c = wave_max(c);
      if (lane == 0) {
        float sc, r;
        scale_from_range(c, K, sc, r);
        table[t] = r;
        int32_t ch = p0.ch + t;
        if (ch >= geom.C) ch -= geom.C;
        // segment t of the tile starts t*seg_vecs - rem vectors after the tile's first vector:
        // inside the tile, and in batch row 0?
        const int64_t start = int64_t(t) * geom.seg_vecs - p0.rem;
        if (start >= 0 && tile * TILE_VECS + start < int64_t(geom.C) * geom.seg_vecs) header[ch] = sc;
      }
    }
  };
  if (MODE == kRangePerVectorLocal && int64_t(blockIdx.x) < full_tiles) {
    LocalFetch lf;
    local_fetch(first_pos, lf);
    local_finish(tile_of(blockIdx.x), first_pos, lf, local_r[0]);
    __syncthreads();
  }

  int buf = 0;
  for (int64_t tile_f = blockIdx.x; tile_f < full_tiles; tile_f += gridDim.x, buf ^= 1) {
    const int64_t tile = tile_of(tile_f);
    // the next tile of this workgroup: one grid stride back inside the reversed part
    const int64_t next_f = tile_f + gridDim.x;
    ChanPos next_pos = first_pos;
    LocalFetch next_lf;
    if (MODE != kOneRange && next_f < full_tiles) {
      if (next_f < rev_tiles) chan_retreat(geom, next_pos, geom.sgrid);
      else next_pos = chan_init(geom, tile_of(next_f) * TILE_VECS);
      if (MODE == kRangePerVectorLocal) local_fetch(next_pos, next_lf);
    }
    ChanPos pos = first_pos;
    if (MODE != kOneRange) chan_advance(geom, pos, mine);
    const int32_t ch0 = first_pos.ch;
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
      float r[VEC];
      if (MODE == kRangePerVectorLocal) {
        int32_t t = pos.ch - ch0;
        if (t < 0) t += geom.C;
        ranges_of_vector<MODE, VEC>(local_r[buf], r_tensor, t, r);
      } else {
        ranges_of_vector<MODE, VEC>(rtab, r_tensor, pos.ch, r);
      }
      if (MODE != kOneRange) chan_advance(geom, pos, geom.s256);
      const int64_t e0 = tile * kTileElems + int64_t(u * kBlock + tid) * VEC;
      float f[VEC];
      widen(raw[u], f);
#pragma unroll
      for (int h = 0; h < QPV; ++h)
        pieces[buf][(u * kBlock + tid) * QPV + h] = quantize4<K, STOCH>(&f[4 * h], &r[4 * h], seed, e0 + 4 * h);
    }
    if (next_f < full_tiles) ask_for_tile(tile_of(next_f));
    if (MODE == kRangePerVectorLocal && next_f < full_tiles)
      local_finish(tile_of(next_f), next_pos, next_lf, local_r[buf ^ 1]);
    first_pos = next_pos;
    __syncthreads();
    const uint4 a = *reinterpret_cast<const uint4*>(&pieces[buf][8 * tid]);
    const uint4 b = *reinterpret_cast<const uint4*>(&pieces[buf][8 * tid + 4]);
    const uint32_t P[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t out[K];
    pack8<K>(P, out);
    store_dwords<K>(payload32 + (tile * kBlock + tid) * K, out);
  }

  // Everything the tile loop did not cover, 8 elements (k bytes) per thread.
  const int64_t groups = (N + 7) / 8;
  uint8_t* payload8 = reinterpret_cast<uint8_t*>(payload32);
  for (int64_t g = slow_first_group + int64_t(blockIdx.x) * kBlock + tid; g < groups;
       g += int64_t(gridDim.x) * kBlock) {
    if (MODE != kOneRange) {
      quantize_group8<T, K, STOCH>(x, payload8, g, N, payload_bytes, seed,
                                   [&](int64_t i) { return rtab[(i % m) / seg_len]; });
    } else {
      quantize_group8<T, K, STOCH>(x, payload8, g, N, payload_bytes, seed, [&](int64_t) { return r_tensor; });
    }
  }
}

// ====================================================================== dequantize (U4+U5)
// Four consecutive codes starting at element index e0 (a multiple of 4): load the one or two
// payload dwords that hold their 4k bits, view them as a big-endian 64-bit window, extract,
// remove the offset by sign extension, multiply by s.
// The payload words of four consecutive codes (hi: the dword holding the first bit; lo: the
// next dword, needed only for widths whose 4-code fields can straddle two dwords).
struct CodeWords {
  uint32_t hi, lo;
};
// e0: element index of the first code (a multiple of 4), relative to a dword-aligned origin.
template <int K>
__device__ __forceinline__ void convert_codes4(CodeWords c, int64_t e0, const float* s, float* out) {
  constexpr int W = 4 * K;
  const int sh = int((e0 * K) & 31);
  const uint64_t win = (uint64_t(__builtin_bswap32(c.hi)) << 32) | __builtin_bswap32(c.lo);
  uint32_t piece = uint32_t(win >> (64 - W - sh));
  // Offset binary -> two's complement: flip the top bit of each k-bit field (k < 8).
  if (K < 8) {
    constexpr uint32_t TOP = (1u << (K - 1)) * ((1u) | (1u << K) | (1u << (2 * K)) | (1u << (3 * K)));
    piece ^= TOP;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int q = __builtin_amdgcn_sbfe(int(piece), K * (3 - e), K);
    out[e] = __fmul_rn(float(q), s[e]);
  }
}
template <int K>
__device__ __forceinline__ void dequant4(const uint32_t* __restrict__ payload32, int64_t e0, const float* s,
                                         float* out) {
  const int64_t w0 = (e0 * K) >> 5;
  CodeWords c;
  c.lo = 0;
  if (32 % (4 * K) != 0) {
    // fields may straddle two dwords: always fetch the pair as one 8-byte load (the vector path
    // stops one 32-element group before the end, so dword w0+1 always exists)
    struct alignas(4) Pair { uint32_t a, b; };
    const Pair pr = *reinterpret_cast<const Pair*>(payload32 + w0);
    c.hi = pr.a;
    c.lo = pr.b;
  } else {
    c.hi = payload32[w0];
  }
  convert_codes4<K>(c, e0, s, out);
}

// Slow path: one element, byte loads guarded by the payload size.
template <int K>
__device__ __forceinline__ float dequant1(const uint8_t* __restrict__ payload, int64_t i, int64_t payload_bytes,
                                          float s) {
  const int64_t bit = i * K;
  const int64_t b0 = bit >> 3;
  const int sh = int(bit & 7);
  uint32_t win = uint32_t(payload[b0]) << 8;
  if (b0 + 1 < payload_bytes) win |= payload[b0 + 1];
  const uint32_t u = (win >> (16 - K - sh)) & ((1u << K) - 1u);
  const int q = (K == 8) ? int(int8_t(u)) : int(u) - (1 << (K - 1));
  return __fmul_rn(float(q), s);
}

template <typename TO, int K, int MODE>
__global__ __launch_bounds__(kBlock) void unpack_dequant_kernel(
    const uint32_t* __restrict__ payload32, const float* __restrict__ header, TO* __restrict__ xhat, int64_t N,
    int64_t fast_vecs, int64_t payload_bytes, ChanGeom geom, int64_t m, int64_t seg_len) {
  constexpr int VEC = Elem<TO>::VEC;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  const float s_tensor = MODE != kOneRange ? 0.0f : header[0];
  ChanPos pos{0, 0};
  if (MODE != kOneRange && v < fast_vecs) pos = chan_init(geom, v);
  for (; v < fast_vecs; v += stride) {
    float s[VEC];
    ranges_of_vector<MODE, VEC>(header, s_tensor, pos.ch, s);
    if (MODE != kOneRange) chan_advance(geom, pos, geom.sgrid);
    float f[VEC];
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) dequant4<K>(payload32, v * VEC + 4 * h, &s[4 * h], &f[4 * h]);
    store_vec(xhat + v * VEC, f);
  }
  const uint8_t* payload8 = reinterpret_cast<const uint8_t*>(payload32);
  for (int64_t i = fast_vecs * VEC + int64_t(blockIdx.x) * kBlock + threadIdx.x; i < N; i += stride) {
    const float s = MODE != kOneRange ? header[(i % m) / seg_len] : s_tensor;
    store_one(xhat + i, dequant1<K>(payload8, i, payload_bytes, s));
  }
}

// Tiled decoder: a workgroup takes the K KiB of payload of one 8192-element tile with 16-byte
// loads that are contiguous across lanes, parks them in local memory, and every thread then
// picks the dword (or dword pair) of each of its output vectors from there; output vector
// j*256 + tid of the tile goes out as one 16-byte streaming store, contiguous across lanes.
// (Reading the payload straight from global memory gives every lane a 4-byte load of which
// half is used at k = 4: the small reads, not the stores, held the plain kernel back.)
// Elements beyond the last whole tile take the scalar path.
template <typename TO, int K, int MODE>
__global__ __launch_bounds__(kBlock) void unpack_dequant_tiled_kernel(
    const uint32_t* __restrict__ payload32, const float* __restrict__ header, TO* __restrict__ xhat, int64_t N,
    int64_t full_tiles, int64_t payload_bytes, ChanGeom geom, int64_t m, int64_t seg_len) {
  constexpr int VEC = Elem<TO>::VEC;
  constexpr int VPT = kTileElems / VEC / kBlock;  // output vectors per thread and tile
  constexpr int TILE_DW = K * (kTileElems / 32);  // payload dwords of a tile
  constexpr int SWEEPS = (TILE_DW + 4 * kBlock - 1) / (4 * kBlock);
  __shared__ __attribute__((aligned(16))) uint32_t tile[2][TILE_DW + 4];  // + one dword a straddling pair may touch
  const int tid = threadIdx.x;
  const float s_tensor = MODE != kOneRange ? 0.0f : header[0];
  ChanPos tile_pos{0, 0};
  if (MODE != kOneRange && full_tiles > 0)
    tile_pos = chan_init(geom, int64_t(blockIdx.x) * (kTileElems / VEC) + tid);
  if (tid < 4) { tile[0][TILE_DW + tid] = 0u; tile[1][TILE_DW + tid] = 0u; }
  int buf = 0;
  for (int64_t t = blockIdx.x; t < full_tiles; t += gridDim.x, buf ^= 1) {
    const uint32_t* src = payload32 + t * TILE_DW;  // 16-byte aligned: TILE_DW is a multiple of 4
#pragma unroll
    for (int w = 0; w < SWEEPS; ++w) {
      const int dw = (w * kBlock + tid) * 4;
      // plain loads: a payload that was written a moment ago is often still in a cache, and
      // streaming loads of such lines cost 9 us per call at the benchmark shape
      if (dw < TILE_DW) *reinterpret_cast<uint4*>(&tile[buf][dw]) = load16(src + dw);
    }
    __syncthreads();  // double buffered: the next tile's writes go to the other half
    ChanPos pos = tile_pos;
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      float s[VEC];
      ranges_of_vector<MODE, VEC>(header, s_tensor, pos.ch, s);
      if (MODE != kOneRange) chan_advance(geom, pos, geom.s256);
      const int vec_in_tile = j * kBlock + tid;
      float f[VEC];
#pragma unroll
      for (int h = 0; h < VEC / 4; ++h) {
        const int e0 = vec_in_tile * VEC + 4 * h;  // element index inside the tile
        const int bit = e0 * K;
        CodeWords c;
        c.hi = tile[buf][bit >> 5];
        c.lo = (32 % (4 * K) != 0) ? tile[buf][(bit >> 5) + 1] : 0u;
        convert_codes4<K>(c, e0, &s[4 * h], &f[4 * h]);
      }
      store_vec(xhat + (t * (kTileElems / VEC) + vec_in_tile) * VEC, f);
    }
    if (MODE != kOneRange) chan_advance(geom, tile_pos, geom.sgrid);
  }
  const uint8_t* payload8 = reinterpret_cast<const uint8_t*>(payload32);
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  for (int64_t i = full_tiles * kTileElems + int64_t(blockIdx.x) * kBlock + tid; i < N; i += stride) {
    const float s = MODE != kOneRange ? header[(i % m) / seg_len] : s_tensor;
    store_one(xhat + i, dequant1<K>(payload8, i, payload_bytes, s));
  }
}

// ============================================================================= host side
ChanStep make_step(int64_t step_vecs, int64_t seg_vecs, int64_t C) {
  ChanStep st;
  st.dr = step_vecs % seg_vecs;
  st.dch = int32_t((step_vecs / seg_vecs) % C);
  return st;
}

template <typename T, int K, int MODE, bool STOCH>
hipError_t launch_quant(const accept_desc& d, const UPlan& p, const T* x, float* header, uint32_t* payload,
                        const float* partials, const float* rtab, hipStream_t s) {
  const int64_t N = p.N;
  const int64_t full_tiles = p.fast ? N / kTileElems : 0;
  const int64_t groups = (N + 7) / 8;
  const int64_t slow_first = full_tiles * (kTileElems / 8);
  const int64_t slow_groups = groups - slow_first;
  int64_t want = full_tiles > (slow_groups + kBlock - 1) / kBlock ? full_tiles : (slow_groups + kBlock - 1) / kBlock;
  if (want < 1) want = 1;
  const int grid = int(want < kQuantGridMax ? want : kQuantGridMax);
  // the reversed tile order needs tile and workgroup index to agree modulo 8
  const int64_t rev_tiles = (grid % 8 == 0) ? (full_tiles & ~int64_t(7)) : 0;
  ChanGeom g{};
  g.seg_vecs = 1;
  g.C = 1;
  if (MODE != kOneRange && p.fast) {
    // per element: the "segments" are single vectors and the "channels" the m / vec vectors of a row
    g.seg_vecs = MODE == kRangePerElement ? 1 : p.seg_len / p.vec;
    g.C = int32_t(MODE == kRangePerElement ? p.m / p.vec : p.C);
    g.s256 = make_step(kBlock, g.seg_vecs, g.C);
    g.sgrid = make_step(int64_t(grid) * (kTileElems / p.vec), g.seg_vecs, g.C);
  }
  const int64_t payload_bytes = (N * K + 7) / 8;
  hipLaunchKernelGGL((quantize_pack_kernel<T, K, MODE, STOCH>), dim3(grid), dim3(kBlock), 0, s, x, payload, header,
                     partials, p.range_grid, rtab, N, full_tiles, rev_tiles, slow_first, payload_bytes, g,
                     LocalRanges{int32_t(d.n * p.cps)}, p.m, p.seg_len, d.seed);
  return hipGetLastError();
}

// ===================================================== comparison layouts (plain kernels)
// ACCEPT_LAYOUT_BATCH and ACCEPT_LAYOUT_UNENCODED: the same quantizer, other ways of laying
// the integers into bytes.  The bit width is a run-time argument here; the reciprocal of every
// range group comes from the table that range_finalize_kernel writes.

// k-bit code of one element, as quantize1 computes it (same arithmetic, run-time k).
__device__ __forceinline__ uint32_t quantize_any(float f, float r, int k, bool stoch, uint64_t seed, int64_t idx) {
  const int half = 1 << (k - 1);
  const uint32_t mask = (1u << k) - 1u;
  const float v = __fmul_rn(f, r);
  if (!stoch) {
    const float t = __fadd_rn(v, kRoundMagic + float(k == 8 ? 0 : half));
    return f32_as_u32(t) & mask;
  }
  const float fl = floorf(v);
  const float pr = __fsub_rn(v, fl);
  const float u = counter_uniform(seed, uint64_t(idx));
  int q = int(fl) + (u < pr ? 1 : 0);
  q = min(max(q, -half), half - 1);
  return (k == 8) ? (uint32_t(q) & 0xFFu) : uint32_t(q + half);
}
// Signed value of a code.
__device__ __forceinline__ int code_to_q(uint32_t code, int k) {
  return k == 8 ? int(int8_t(code)) : int(code) - (1 << (k - 1));
}

// UNENCODED: byte i = q_i (two's complement).  Four elements per thread and step, the last
// N % 4 elements one per thread.
template <typename T>
__global__ __launch_bounds__(kBlock) void quantize_bytes_kernel(const T* __restrict__ x,
                                                                const float* __restrict__ rtab,
                                                                uint8_t* __restrict__ payload, int64_t N, int64_t m,
                                                                int64_t seg_len, int k, int stoch, uint64_t seed) {
  const int64_t quads = N / 4;
  const bool one = seg_len == m;  // a single range group
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  for (int64_t u = gtid; u < quads; u += stride) {
    float f[4];
    load_quad<T>(x + 4 * u, f);
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t i = 4 * u + e;
      const float r = one ? rtab[0] : rtab[(i % m) / seg_len];
      w |= (uint32_t(code_to_q(quantize_any(f[e], r, k, stoch != 0, seed, i), k)) & 0xFFu) << (8 * e);
    }
    *reinterpret_cast<uint32_t*>(payload + 4 * u) = w;
  }
  const int64_t i = quads * 4 + gtid;
  if (i < N) {
    const float r = one ? rtab[0] : rtab[(i % m) / seg_len];
    payload[i] = uint8_t(code_to_q(quantize_any(load_one(x + i), r, k, stoch != 0, seed, i), k));
  }
}

template <typename TO>
__global__ __launch_bounds__(kBlock) void dequant_bytes_kernel(const uint8_t* __restrict__ payload,
                                                               const float* __restrict__ header,
                                                               TO* __restrict__ xhat, int64_t N, int64_t m,
                                                               int64_t seg_len) {
  const int64_t quads = N / 4;
  const bool one = seg_len == m;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  for (int64_t u = gtid; u < quads; u += stride) {
    const uint32_t w = *reinterpret_cast<const uint32_t*>(payload + 4 * u);
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t i = 4 * u + e;
      const float s = one ? header[0] : header[(i % m) / seg_len];
      f[e] = __fmul_rn(float(int(int8_t(w >> (8 * e)))), s);
    }
    store_quad<TO>(xhat + 4 * u, f);
  }
  const int64_t i = quads * 4 + gtid;
  if (i < N) {
    const float s = one ? header[0] : header[(i % m) / seg_len];
    store_one(xhat + i, __fmul_rn(float(int(int8_t(payload[i]))), s));
  }
}

// BATCH: byte g*m + j = codes of rows g*per .. g*per+per-1 of column j (per = 8/k), first row
// in the most significant bits.  With m % 4 == 0 a thread takes four columns (16-byte row
// loads, one dword store); otherwise one byte per thread.
template <typename T>
__global__ __launch_bounds__(kBlock) void quantize_batch_kernel(const T* __restrict__ x,
                                                                const float* __restrict__ rtab,
                                                                uint8_t* __restrict__ payload, int64_t n, int64_t m,
                                                                int64_t seg_len, int k, int stoch, uint64_t seed) {
  const int per = 8 / k;
  const int64_t G = (n + per - 1) / per;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (m % 4 == 0) {
    const int64_t m4 = m / 4;
    for (int64_t u = gtid; u < G * m4; u += stride) {
      const int64_t g = u / m4, j0 = (u - g * m4) * 4;
      float r[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = rtab[(j0 + e) / seg_len];
      uint32_t w = 0;
      for (int i = 0; i < per; ++i) {
        const int64_t row = g * per + i;
        if (row >= n) break;
        float f[4];
        load_quad<T>(x + row * m + j0, f);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          w |= quantize_any(f[e], r[e], k, stoch != 0, seed, row * m + j0 + e) << (8 * e + k * (per - 1 - i));
      }
      *reinterpret_cast<uint32_t*>(payload + g * m + j0) = w;
    }
  } else {
    for (int64_t u = gtid; u < G * m; u += stride) {
      const int64_t g = u / m, j = u - g * m;
      const float r = rtab[j / seg_len];
      uint32_t b = 0;
      for (int i = 0; i < per; ++i) {
        const int64_t row = g * per + i;
        if (row >= n) break;
        b |= quantize_any(load_one(x + row * m + j), r, k, stoch != 0, seed, row * m + j) << (k * (per - 1 - i));
      }
      payload[u] = uint8_t(b);
    }
  }
}

template <typename TO>
__global__ __launch_bounds__(kBlock) void dequant_batch_kernel(const uint8_t* __restrict__ payload,
                                                               const float* __restrict__ header,
                                                               TO* __restrict__ xhat, int64_t n, int64_t m,
                                                               int64_t seg_len, int k) {
  const int per = 8 / k;
  const uint32_t mask = (1u << k) - 1u;
  const int64_t G = (n + per - 1) / per;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (m % 4 == 0) {
    const int64_t m4 = m / 4;
    for (int64_t u = gtid; u < G * m4; u += stride) {
      const int64_t g = u / m4, j0 = (u - g * m4) * 4;
      const uint32_t w = *reinterpret_cast<const uint32_t*>(payload + g * m + j0);
      float s[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] = header[(j0 + e) / seg_len];
      for (int i = 0; i < per; ++i) {
        const int64_t row = g * per + i;
        if (row >= n) break;
        float f[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          f[e] = __fmul_rn(float(code_to_q((w >> (8 * e + k * (per - 1 - i))) & mask, k)), s[e]);
        store_quad<TO>(xhat + row * m + j0, f);
      }
    }
  } else {
    for (int64_t u = gtid; u < G * m; u += stride) {
      const int64_t g = u / m, j = u - g * m;
      const uint32_t b = payload[u];
      const float s = header[j / seg_len];
      for (int i = 0; i < per; ++i) {
        const int64_t row = g * per + i;
        if (row >= n) break;
        store_one(xhat + row * m + j, __fmul_rn(float(code_to_q((b >> (k * (per - 1 - i))) & mask, k)), s));
      }
    }
  }
}

int plain_grid(int64_t units) {
  int64_t blocks = (units + kBlock - 1) / kBlock;
  if (blocks < 1) blocks = 1;
  return int(blocks < 8192 ? blocks : 8192);
}

template <typename T, int K>
hipError_t launch_quant_k(const accept_desc& d, const UPlan& p, const T* x, float* header, uint32_t* payload,
                          const float* partials, const float* rtab, hipStream_t s) {
  const bool stoch = d.rounding == ACCEPT_ROUND_STOCHASTIC;
  if (p.mode == U_TENSOR) {
    return stoch ? launch_quant<T, K, kOneRange, true>(d, p, x, header, payload, partials, rtab, s)
                 : launch_quant<T, K, kOneRange, false>(d, p, x, header, payload, partials, rtab, s);
  }
  if (p.per_element) {
    return stoch ? launch_quant<T, K, kRangePerElement, true>(d, p, x, header, payload, partials, rtab, s)
                 : launch_quant<T, K, kRangePerElement, false>(d, p, x, header, payload, partials, rtab, s);
  }
  if (p.local_ranges) {
    return stoch ? launch_quant<T, K, kRangePerVectorLocal, true>(d, p, x, header, payload, partials, rtab, s)
                 : launch_quant<T, K, kRangePerVectorLocal, false>(d, p, x, header, payload, partials, rtab, s);
  }
  return stoch ? launch_quant<T, K, kRangePerVector, true>(d, p, x, header, payload, partials, rtab, s)
               : launch_quant<T, K, kRangePerVector, false>(d, p, x, header, payload, partials, rtab, s);
}

template <typename T>
hipError_t compress_typed(const accept_desc& d, const UPlan& p, const T* x, float* header, uint32_t* payload,
                          void* ws, hipStream_t s, StageTimer* tm) {
  float* partials = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + kCtrlBytes);
  float* rtab = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + p.off_rtab);
  mark(tm, s);
  if (p.mode == U_TENSOR) {
    hipLaunchKernelGGL((range_tensor_kernel<T>), dim3(p.range_grid), dim3(kBlock), 0, s, x, p.N, partials);
  } else if (p.mode == U_SEGMENTED) {
    const int64_t tiles = (p.N + kTileElems - 1) / kTileElems;  // below 2^31: N is at most 2^40
    hipLaunchKernelGGL((range_segments_kernel<T>), dim3(unsigned(tiles)), dim3(kBlock), 0, s, x, p.items, p.cps,
                       p.seg_len / p.vec, p.chunk_vecs, d.n, p.C, partials);
  } else {
    const dim3 grid(unsigned(p.col_grid_x), unsigned(p.col_grid_y));
    if (p.m % Elem<T>::VEC == 0)
      hipLaunchKernelGGL((range_columns_kernel<T, Elem<T>::VEC>), grid, dim3(kBlock), 0, s, x, d.n, p.m, p.col_tx,
                         partials);
    else
      hipLaunchKernelGGL((range_columns_kernel<T, 1>), grid, dim3(kBlock), 0, s, x, d.n, p.m, p.col_tx, partials);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  mark(tm, s);
  const bool plain = d.layout != ACCEPT_LAYOUT_PACKED;
  if (p.mode == U_GENERIC) {
    hipLaunchKernelGGL(range_columns_finalize_kernel, dim3(unsigned(p.C)), dim3(kBlock), 0, s, partials, p.m, p.seg_len,
                       p.col_grid_y, d.bits, header, rtab);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    mark(tm, s);
  } else if ((p.mode != U_TENSOR || plain) && !(p.local_ranges && !plain)) {
    // the per-tensor pass leaves range_grid maxima: one row, one channel, range_grid chunks
    const int64_t rows = p.mode == U_SEGMENTED ? d.n : 1;
    const int64_t cps = p.mode == U_SEGMENTED ? p.cps : p.range_grid;
    hipLaunchKernelGGL(range_finalize_kernel, dim3(unsigned(p.C)), dim3(kWave), 0, s, partials, rows * cps, d.bits,
                       header, rtab);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    mark(tm, s);
  }
  if (plain) {
    uint8_t* pl = reinterpret_cast<uint8_t*>(payload);
    const int stoch = d.rounding == ACCEPT_ROUND_STOCHASTIC ? 1 : 0;
    if (d.layout == ACCEPT_LAYOUT_UNENCODED) {
      hipLaunchKernelGGL((quantize_bytes_kernel<T>), dim3(plain_grid(p.N / 4 + 4)), dim3(kBlock), 0, s, x, rtab, pl,
                         p.N, p.m, p.seg_len, d.bits, stoch, d.seed);
    } else {
      const int per = 8 / d.bits;
      const int64_t G = (d.n + per - 1) / per;
      hipLaunchKernelGGL((quantize_batch_kernel<T>), dim3(plain_grid(p.m % 4 == 0 ? G * (p.m / 4) : G * p.m)),
                         dim3(kBlock), 0, s, x, rtab, pl, d.n, p.m, p.seg_len, d.bits, stoch, d.seed);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    mark(tm, s);
    return hipSuccess;
  }
  switch (d.bits) {
    case 2: e = launch_quant_k<T, 2>(d, p, x, header, payload, partials, rtab, s); break;
    case 3: e = launch_quant_k<T, 3>(d, p, x, header, payload, partials, rtab, s); break;
    case 4: e = launch_quant_k<T, 4>(d, p, x, header, payload, partials, rtab, s); break;
    case 5: e = launch_quant_k<T, 5>(d, p, x, header, payload, partials, rtab, s); break;
    case 6: e = launch_quant_k<T, 6>(d, p, x, header, payload, partials, rtab, s); break;
    case 7: e = launch_quant_k<T, 7>(d, p, x, header, payload, partials, rtab, s); break;
    case 8: e = launch_quant_k<T, 8>(d, p, x, header, payload, partials, rtab, s); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  mark(tm, s);
  return hipSuccess;
}

template <typename TO, int K, int MODE>
hipError_t launch_dequant(const accept_desc& d, const float* header, const uint32_t* payload, TO* xhat,
                          hipStream_t s) {
  constexpr int VEC = Elem<TO>::VEC;
  const int64_t N = d.n * d.m;
  const int64_t C = d.channels > 1 ? d.channels : 1;
  const int64_t seg_len = d.m / C;
  // The vector path covers whole groups of 32 elements (k whole dwords), so that no dword
  // load reaches past the payload; per channel it also needs vectors that stay in a segment.
  const bool fast = MODE != kRangePerVector || (seg_len % VEC == 0);
  // widths whose 4-code fields straddle dwords read dword pairs: keep one group in reserve
  const int64_t groups32 = (32 % (4 * K) != 0) ? (N / 32 > 0 ? N / 32 - 1 : 0) : N / 32;
  const int64_t fast_vecs = fast ? groups32 * (32 / VEC) : 0;
  const int64_t work = fast_vecs > (N - fast_vecs * VEC) ? fast_vecs : (N - fast_vecs * VEC);
  int64_t blocks = (work + kBlock - 1) / kBlock;
  if (blocks < 1) blocks = 1;
  const int grid = int(blocks < kDequantGridMax ? blocks : kDequantGridMax);
  ChanGeom g{};
  g.seg_vecs = 1;
  g.C = 1;
  if (MODE != kOneRange && fast) {
    g.seg_vecs = MODE == kRangePerElement ? 1 : seg_len / VEC;
    g.C = int32_t(MODE == kRangePerElement ? d.m / VEC : C);
    g.sgrid = make_step(int64_t(grid) * kBlock, g.seg_vecs, g.C);
    g.s256 = g.sgrid;
  }
  const int64_t payload_bytes = (N * K + 7) / 8;
  const int64_t full_tiles = fast ? N / kTileElems : 0;
  if (full_tiles > 0) {
    const int64_t tail = N - full_tiles * kTileElems;
    int64_t want = full_tiles > (tail + kBlock - 1) / kBlock ? full_tiles : (tail + kBlock - 1) / kBlock;
    const int tgrid = int(want < kDequantGridMax ? want : kDequantGridMax);
    if (MODE != kOneRange) {
      g.s256 = make_step(kBlock, g.seg_vecs, g.C);
      g.sgrid = make_step(int64_t(tgrid) * (kTileElems / VEC), g.seg_vecs, g.C);
    }
    hipLaunchKernelGGL((unpack_dequant_tiled_kernel<TO, K, MODE>), dim3(tgrid), dim3(kBlock), 0, s, payload, header,
                       xhat, N, full_tiles, payload_bytes, g, d.m, seg_len);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((unpack_dequant_kernel<TO, K, MODE>), dim3(grid), dim3(kBlock), 0, s, payload, header, xhat, N,
                     fast_vecs, payload_bytes, g, d.m, seg_len);
  return hipGetLastError();
}

template <typename TO>
hipError_t decompress_typed(const accept_desc& d, const float* header, const uint32_t* payload, TO* xhat,
                            hipStream_t s) {
  if (d.layout != ACCEPT_LAYOUT_PACKED) {
    const uint8_t* pl = reinterpret_cast<const uint8_t*>(payload);
    const int64_t N = d.n * d.m;
    const int64_t seg_len = d.m / (d.channels > 1 ? d.channels : 1);
    if (d.layout == ACCEPT_LAYOUT_UNENCODED) {
      hipLaunchKernelGGL((dequant_bytes_kernel<TO>), dim3(plain_grid(N / 4 + 4)), dim3(kBlock), 0, s, pl, header,
                         xhat, N, d.m, seg_len);
    } else {
      const int per = 8 / d.bits;
      const int64_t G = (d.n + per - 1) / per;
      hipLaunchKernelGGL((dequant_batch_kernel<TO>), dim3(plain_grid(d.m % 4 == 0 ? G * (d.m / 4) : G * d.m)),
                         dim3(kBlock), 0, s, pl, header, xhat, d.n, d.m, seg_len, d.bits);
    }
    return hipGetLastError();
  }
  // channels-last (every element of a row its own channel) with rows of whole vectors: one range per element
  // (the scales are then read as 16-byte vectors: a header that is only 4-byte aligned takes the plain path)
  const bool per_element = d.channels > 1 && d.channels == d.m && d.m % Elem<TO>::VEC == 0 &&
                           (reinterpret_cast<uintptr_t>(header) & 15u) == 0;
  const int mode = d.channels > 1 ? (per_element ? kRangePerElement : kRangePerVector) : kOneRange;
#define ACCEPT_DQ(KK)                                                                                   \
  case KK:                                                                                              \
    return mode == kRangePerElement  ? launch_dequant<TO, KK, kRangePerElement>(d, header, payload, xhat, s) \
           : mode == kRangePerVector ? launch_dequant<TO, KK, kRangePerVector>(d, header, payload, xhat, s)  \
                                     : launch_dequant<TO, KK, kOneRange>(d, header, payload, xhat, s);
  switch (d.bits) {
    ACCEPT_DQ(2) ACCEPT_DQ(3) ACCEPT_DQ(4) ACCEPT_DQ(5) ACCEPT_DQ(6) ACCEPT_DQ(7) ACCEPT_DQ(8)
    default: return hipErrorInvalidValue;
  }
#undef ACCEPT_DQ
}

}  // namespace

UPlan make_uplan(const accept_desc& d) {
  UPlan p{};
  p.N = d.n * d.m;
  p.m = d.m;
  p.C = d.channels > 1 ? d.channels : 1;
  p.seg_len = d.m / p.C;
  p.vec = d.in_dtype == ACCEPT_BF16 ? 8 : 4;
  p.cps = 1;
  p.chunk_vecs = 1;
  p.items = 0;
  p.range_grid = 1;
  size_t partial_bytes;
  if (p.C == 1) {
    p.mode = U_TENSOR;
    p.fast = true;
    int64_t blocks = p.N / kTileElems;  // one tile per workgroup and round
    if (blocks < 1) blocks = 1;
    p.range_grid = int(blocks < kRangeGridMax ? blocks : kRangeGridMax);
    partial_bytes = size_t(4096) * sizeof(float);
  } else if (p.seg_len % p.vec == 0 && p.seg_len >= 512) {
    p.mode = U_SEGMENTED;
    p.fast = true;
    const int64_t seg_vecs = p.seg_len / p.vec;
    const int64_t max_chunk = kTileElems / p.vec;  // vectors one wavefront reduces: at most a tile of the quantize pass
    p.cps = (seg_vecs + max_chunk - 1) / max_chunk;
    p.chunk_vecs = (seg_vecs + p.cps - 1) / p.cps;
    p.items = d.n * p.C * p.cps;
    partial_bytes = size_t(p.items) * sizeof(float);
    // A tensor of whole tiles with few partial maxima per channel: the quantize pass finishes the
    // ranges of each tile's channels itself (no U1b kernel between the passes).
    p.local_ranges = p.N % kTileElems == 0 && p.seg_len >= kLocalMinSegment && d.n * p.cps <= 128 &&
                     p.C * d.n * p.cps < (int64_t(1) << 31) && d.layout == ACCEPT_LAYOUT_PACKED;
  } else {
    p.mode = U_GENERIC;
    // channels-last (one element per segment) with rows of whole vectors: the quantizer's fast
    // path with one range per element
    p.per_element = p.seg_len == 1 && d.m % p.vec == 0;
    p.fast = (p.seg_len % p.vec == 0) || p.per_element;
    // column pass: threads own vectors of columns when every row keeps them aligned, else columns
    const int64_t ncv = (d.m % p.vec == 0) ? d.m / p.vec : d.m;
    int tx = 1;
    while (tx < kBlock && tx < ncv) tx *= 2;
    p.col_tx = tx;
    const int64_t ty = kBlock / tx;
    const int64_t gx = (ncv + tx - 1) / tx;
    int64_t gy = (d.n + ty - 1) / ty;                      // at most one row per thread row
    const int64_t want = gx >= 2048 ? 1 : 2048 / gx;       // about 2048 workgroups in all
    if (gy > want) gy = want;
    const int64_t cap = (int64_t(16) << 20) / d.m;         // at most 64 MiB of column maxima
    if (gy > cap) gy = cap;
    if (gy < 1) gy = 1;
    if (gy > 65535) gy = 65535;
    p.col_grid_x = gx;
    p.col_grid_y = int(gy);
    partial_bytes = size_t(gy) * size_t(d.m) * sizeof(float);
  }
  p.off_rtab = kCtrlBytes + (partial_bytes + 255) / 256 * 256;
  p.bytes = p.off_rtab + (size_t(p.C) * sizeof(float) + 255) / 256 * 256;
  return p;
}

hipError_t launch_uniform_compress(const accept_desc& d, const UPlan& p, const void* x, void* header, void* payload,
                                   void* ws, hipStream_t s, StageTimer* tm) {
  if (d.in_dtype == ACCEPT_BF16)
    return compress_typed<bf16_t>(d, p, static_cast<const bf16_t*>(x), static_cast<float*>(header),
                                  static_cast<uint32_t*>(payload), ws, s, tm);
  return compress_typed<float>(d, p, static_cast<const float*>(x), static_cast<float*>(header),
                               static_cast<uint32_t*>(payload), ws, s, tm);
}

hipError_t launch_uniform_decompress(const accept_desc& d, const void* header, const void* payload, void* xhat,
                                     hipStream_t s, StageTimer* tm) {
  mark(tm, s);
  hipError_t e;
  if (d.out_dtype == ACCEPT_BF16)
    e = decompress_typed<bf16_t>(d, static_cast<const float*>(header), static_cast<const uint32_t*>(payload),
                                 static_cast<bf16_t*>(xhat), s);
  else
    e = decompress_typed<float>(d, static_cast<const float*>(header), static_cast<const uint32_t*>(payload),
                                static_cast<float*>(xhat), s);
  if (e != hipSuccess) return e;
  mark(tm, s);
  return hipSuccess;
}

}  // namespace accept
