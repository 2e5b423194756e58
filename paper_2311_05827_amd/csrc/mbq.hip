// Scheme M on gfx950: multi-bit quantization x ~ B alpha with batch bit planes (paper
// paragraphs "Forward Quantizer", "Forward Encoder", "Forward Decoder", "Forward
// Dequantizer"; eqs. (MBQ), (alpha solution), (alpha update), (biased error)).
//
// Work item = 8 batch rows (one row group) x VEC adjacent columns.  The eight row loads of
// a wavefront are each contiguous across lanes; the 8 x k bit transpose the encoder needs
// happens in registers (a per-level table holds each sign pattern "spread" to one bit per
// byte, and eight shift-or steps build the k plane bytes of a column), so the encoder needs
// no LDS exchange and its k*VEC output bytes per lane are contiguous across lanes.  The
// least-squares sums ride along in the same pass: bit counts come from popcounts of the
// finished plane bytes, B^T x from multiply-adds with the 0/1 plane bits.
#include "common.hpp"

namespace accept {

namespace {

// Launch-shape constants; the -D overrides exist for tuning sweeps only.
#ifndef ACCEPT_ENCODE_GRID
#define ACCEPT_ENCODE_GRID 768
#endif
#ifndef ACCEPT_ENCODE_WAVES
#define ACCEPT_ENCODE_WAVES 2  // wavefronts per SIMD the encode kernel is compiled for
#endif
#ifndef ACCEPT_ENCODE_GROUP
#define ACCEPT_ENCODE_GROUP 4  // elements whose table lookups are issued together (at least one row)
#endif
#ifndef ACCEPT_DECODE_GRID
#define ACCEPT_DECODE_GRID 8192
#endif
constexpr int kEncodeGridMax = ACCEPT_ENCODE_GRID;  // also the number of partial-sum records
constexpr int kDecodeGridMax = ACCEPT_DECODE_GRID;
constexpr int kInitGrid = 1024;
static_assert(kEncodeGridMax <= 2048, "the workspace holds at most 2048 records");

template <int NDW>
struct alignas((NDW % 4 == 0) ? 16 : (NDW % 2 == 0) ? 8 : 4) Dwords {
  uint32_t v[NDW];
};

__host__ __device__ constexpr int nstat_of(int k) { return k + 1 + k + k * (k - 1) / 2; }

// Position of a work item (row group g, column vector jv), advanced without divisions.
struct ItemPos {
  int64_t g, jv;
};
struct ItemStep {
  int64_t dg, dj;
};
__device__ __forceinline__ void item_advance(ItemPos& p, const ItemStep& st, int64_t ipg) {
  p.jv += st.dj;
  p.g += st.dg;
  if (p.jv >= ipg) { p.jv -= ipg; p.g += 1; }
}

// M1: the 2^k levels sum_j(+-alpha_j) (float32 sums in the order j = 0..k-1 from 0), sorted
// ascending with ties by pattern.  Thread `pat` computes its level and its rank; on return
// lv_sorted[rank] and pat_sorted[rank] are filled (after the caller's barrier).
template <int K>
__device__ __forceinline__ void build_levels(const float* __restrict__ alpha, float* lv_raw, float* lv_sorted,
                                             uint32_t* pat_sorted) {
  constexpr int P = 1 << K;
  const int pat = threadIdx.x;
  float lv = 0.0f;
  if (pat < P) {
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const float a = alpha[j];
      lv = __fadd_rn(lv, ((pat >> j) & 1) ? a : -a);
    }
    lv_raw[pat] = lv;
  }
  __syncthreads();
  if (pat < P) {
    int rank = 0;
    for (int q = 0; q < P; ++q) {
      const float o = lv_raw[q];
      rank += (o < lv || (o == lv && q < pat)) ? 1 : 0;
    }
    lv_sorted[rank] = lv;
    pat_sorted[rank] = uint32_t(pat);
  }
  __syncthreads();
}

// ================================================================ encode + sums (M1..M4)
// M2 without a per-element binary search.  The top 12 bits of a float32 (sign, exponent, three
// mantissa bits) name a bucket, i.e. an interval of reals.  For every bucket a table holds
// lo = number of thresholds below the whole bucket; the element's position among the sorted
// levels is then lo + #{c < maxcnt : x > tau[lo + c]}, where maxcnt is the largest number of
// thresholds that fall inside any one bucket (1 for well separated levels) and tau is padded
// with +inf.  The float compares decide; the table only says where to start, so the result is
// exactly #{i : x > tau_i}.
#ifndef ACCEPT_LUT_BITS
#define ACCEPT_LUT_BITS 12
#endif
constexpr int kLutBits = ACCEPT_LUT_BITS;
constexpr int kLutSize = 1 << kLutBits;

template <int K>
struct EncodeTables {
  static constexpr int P = 1 << K;
  static constexpr int NW = (K + 3) / 4;  // spread words per level
  float lv_raw[P];
  float lv_sorted[P];
  uint32_t pat_sorted[P];
  float tau[3 * P];                        // P-1 thresholds, then +inf padding (the windowed search reads past them)
  uint32_t spread[P * NW];                 // per sorted level: bit p of the sign pattern at bit 8*(p%4) of word p/4
  // k <= 4 only: row lo = {tau[lo] (or +inf), spread[lo]}, so that one 8-byte read at lo*8 and one
  // 4-byte read at lo*8 + 12 (= spread[lo+1]) give everything an element needs (two 8-byte reads
  // and one 4-byte read when a bucket may hold two thresholds)
  alignas(8) uint32_t pair[2 * (P + 2)];
  static constexpr int LUT_SHIFT = (K <= 4) ? 3 : 0;  // bucket table entries are lo << LUT_SHIFT
  alignas(4) uint8_t lut[kLutSize];
  int maxcnt;
};

// Smallest value of bucket b (bit patterns b << shift .. (b << shift) | low-ones); buckets of
// negative values run backwards in bit order.
__device__ __forceinline__ float bucket_vmin(int b) {
  const uint32_t lo_bits = uint32_t(b) << (32 - kLutBits);
  const uint32_t hi_bits = lo_bits | ((1u << (32 - kLutBits)) - 1u);
  return u32_as_f32((b >> (kLutBits - 1)) ? hi_bits : lo_bits);
}

template <int K>
__device__ __forceinline__ void build_encode_tables(const float* __restrict__ alpha_prev, EncodeTables<K>& tb) {
  using TB = EncodeTables<K>;
  constexpr int P = TB::P;
  constexpr int PER = kLutSize / kBlock;  // consecutive buckets per thread
  static_assert(kLutSize % (4 * kBlock) == 0, "each thread writes whole dwords of the bucket table");
  const int tid = threadIdx.x;
  if (tid == 0) tb.maxcnt = 1;
  build_levels<K>(alpha_prev, tb.lv_raw, tb.lv_sorted, tb.pat_sorted);
  for (int i = tid; i < 3 * P; i += kBlock)
    tb.tau[i] = (i < P - 1) ? __fmul_rn(0.5f, __fadd_rn(tb.lv_sorted[i], tb.lv_sorted[i + 1])) : __builtin_inff();
  if (tid < P) {
    const uint32_t pat = tb.pat_sorted[tid];
#pragma unroll
    for (int w = 0; w < TB::NW; ++w) {
      uint32_t sp = 0;
#pragma unroll
      for (int bb = 0; bb < 4; ++bb)
        if (4 * w + bb < K) sp |= ((pat >> (4 * w + bb)) & 1u) << (8 * bb);
      tb.spread[tid * TB::NW + w] = sp;
    }
  }
  __syncthreads();
  if (K <= 4 && tid <= P + 1) {
    tb.pair[2 * tid] = f32_as_u32(tb.tau[tid]);                  // tau[P-1], tau[P], tau[P+1] are +inf
    tb.pair[2 * tid + 1] = tid < P ? tb.spread[tid] : 0u;
  }
  // lo(b) = #{tau_i < smallest value of bucket b}.  tau[0..P-1) is sorted and tau[P-1] = +inf, so a
  // branch-free binary search over P entries finds it.  A thread owns PER consecutive buckets
  // (one more is evaluated for the count below) and writes them four to a dword.
  // Thresholds inside bucket b = lo(value-order successor of b) - lo(b); the successor is b+1 on
  // the positive side and b-1 on the negative side (bucket kLutSize/2 is followed by bucket 0).
  // Buckets of NaN bit patterns get lo = 0, which makes their differences <= 0: ignored.
  int mymax = 0;
  uint32_t* lut32 = reinterpret_cast<uint32_t*>(tb.lut);
  constexpr int CH = 8;  // buckets per step: bounds the registers this prologue needs
  static_assert(PER % CH == 0, "bucket chunks");
#pragma nounroll
  for (int c0 = 0; c0 < PER; c0 += CH) {
    const int b0 = tid * PER + c0;
    const bool neg = b0 >= kLutSize / 2;
    int lo[CH + 2];  // lo[j+1] belongs to bucket b0 + j; lo[0] and lo[CH+1] are the neighbours
#pragma unroll
    for (int j = -1; j <= CH; ++j) {
      int b = b0 + j;
      if (b < 0) b = kLutSize / 2;          // predecessor of bucket 0 in value order is -0's bucket
      if (b >= kLutSize) b = kLutSize - 1;  // no bucket beyond the last: reuse it (difference 0)
      const float vmin = bucket_vmin(b);
      int l = 0;
#pragma unroll
      for (int s = P >> 1; s >= 1; s >>= 1) l += (tb.tau[l + s - 1] < vmin) ? s : 0;
      lo[j + 1] = l;
    }
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      // positive side: the successor is the next bucket; negative side: the previous one, except
      // that the -0 bucket (kLutSize/2) is followed by bucket 0: that pair is counted below
      int cnt = neg ? lo[j] - lo[j + 1] : lo[j + 2] - lo[j + 1];
      if (neg && b0 + j == kLutSize / 2) cnt = 0;
      if (!neg && b0 + j == kLutSize / 2 - 1) cnt = 0;  // top positive bucket: NaN patterns, no successor
      mymax = cnt > mymax ? cnt : mymax;
    }
    if (b0 == 0) {
      // thresholds inside the -0 bucket: lo(bucket 0) - lo(bucket kLutSize/2); lo[0] is that bucket
      const int cnt = lo[1] - lo[0];
      mymax = cnt > mymax ? cnt : mymax;
    }
#pragma unroll
    for (int j = 0; j < CH; j += 4)
      lut32[(b0 + j) / 4] = (uint32_t(lo[j + 1]) | (uint32_t(lo[j + 2]) << 8) | (uint32_t(lo[j + 3]) << 16) |
                             (uint32_t(lo[j + 4]) << 24))
                            << TB::LUT_SHIFT;  // lo < 32 when shifted by 3: no carry between bytes
  }
  if (mymax > 1) atomicMax(&tb.maxcnt, mymax);
  __syncthreads();
}

// Sum of NS per-thread float64 values over the 256 threads of a workgroup, in a fixed order
// (so the result does not depend on timing): the values go to local memory one statistic per
// row, 16 threads per statistic add 16 consecutive entries each, one thread adds those 16
// partial sums.  Far cheaper than NS butterflies of 64-bit lane exchanges.  buf holds
// kStatChunk rows; more statistics than that take several passes.  On return thread s < NS
// holds total s in its return value (other threads: unspecified).
constexpr int kStatChunk = 16;
struct StatScratch {
  double v[kStatChunk][kBlock];
  double part[kStatChunk][16];
};
template <int NS>
__device__ __forceinline__ double block_sum_stats(const double (&sv)[NS], StatScratch& buf) {
  static_assert(kBlock == 256, "16 threads x 16 entries per statistic");
  const int tid = threadIdx.x;
  double mine = 0.0;
#pragma unroll
  for (int c0 = 0; c0 < NS; c0 += kStatChunk) {
    constexpr int kAll = kStatChunk;
    const int nc = (NS - c0) < kAll ? (NS - c0) : kAll;
    if (c0 > 0) __syncthreads();  // the previous pass has been read
#pragma unroll
    for (int s = 0; s < kAll; ++s)
      if (c0 + s < NS) buf.v[s][tid] = sv[c0 + s];
    __syncthreads();
    {
      const int s = tid >> 4, part = tid & 15;
      if (s < nc) {
        const double* src = &buf.v[s][part * 16];
        double a = src[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) a += src[i];
        buf.part[s][part] = a;
      }
    }
    __syncthreads();
    if (tid >= c0 && tid < c0 + nc) {
      const double* src = buf.part[tid - c0];
      double a = src[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) a += src[i];
      mine = a;
    }
  }
  return mine;
}

// Statistics carried by one thread.
template <int K>
struct EncodeStats {
  static constexpr int NPAIR = K * (K - 1) / 2;
  double H[K];      // sum of x over the +1 entries of plane p
  double Sx;        // 1^T x
  uint32_t cnt[K];  // +1 signs per plane
  uint32_t dis[NPAIR > 0 ? NPAIR : 1];  // elements whose planes p<q disagree
};

// M2 for one element, any K: sorted-level position via the bucket table, then the level's spread
// sign pattern.  Adds x to the running float32 sums: S_x always, A_p where plane p is +1
// (byte p of the spread word is 0 or 1; converting it to float and using a fused
// multiply-add gives x*1 or x*0 exactly, so each step rounds like a plain add).
template <int K>
__device__ __forceinline__ void accumulate_elem(float x, const uint32_t (&sp)[(K + 3) / 4], float (&a32)[K],
                                                float& sx32) {
  sx32 = __fadd_rn(sx32, x);
#pragma unroll
  for (int p = 0; p < K; ++p) a32[p] = __fmaf_rn(x, float((sp[p / 4] >> (8 * (p % 4))) & 0xFFu), a32[p]);
}

template <int K>
__device__ __forceinline__ void encode_elem(const EncodeTables<K>& tb, float x, int maxcnt,
                                            uint32_t (&sp)[(K + 3) / 4], float (&a32)[K], float& sx32) {
  using TB = EncodeTables<K>;
  const int lo = tb.lut[f32_as_u32(x) >> (32 - kLutBits)] >> TB::LUT_SHIFT;
  // #{c < maxcnt : x > tau[lo + c]}: the thresholds are sorted, so the true compares form a
  // prefix of tau[lo ..]; its length (at most maxcnt) is found by a branch-free binary search
  // over a window of 2*top - 1 >= maxcnt entries, top = the largest power of two <= maxcnt.
  // lo <= P-1 and the window is shorter than 2P: every read stays inside tau[3P).
  int cnt = 0;
#pragma nounroll
  for (int step = 1 << (31 - __clz(maxcnt)); step >= 1; step >>= 1)
    cnt += (x > tb.tau[lo + cnt + step - 1]) ? step : 0;
  const int idx = lo + cnt;
#pragma unroll
  for (int w = 0; w < TB::NW; ++w) sp[w] = tb.spread[idx * TB::NW + w];
  accumulate_elem<K>(x, sp, a32, sx32);
}

// M2 for NE elements.  MC = 1 or 2: no bucket holds more than MC thresholds (K <= 4 then takes
// everything an element needs from the pair table: the level is lo .. lo+MC); MC = 0: any
// number, maxcnt.  The pair-table form is written in three passes over the elements (bucket
// reads, row reads, selects and sums), so that the local-memory latencies of the NE elements
// overlap whatever order the instruction scheduler keeps.
template <int K, int MC, int NE>
__device__ __forceinline__ void encode_group(const EncodeTables<K>& tb, const float (&xs)[NE], int maxcnt,
                                             uint32_t (&sp)[NE][(K + 3) / 4], float (&a32)[K], float& sx32) {
  if constexpr (K <= 4 && (MC == 1 || MC == 2)) {
    const char* pair = reinterpret_cast<const char*>(tb.pair);
    uint32_t off[NE];  // lo * 8
#pragma unroll
    for (int e = 0; e < NE; ++e) off[e] = tb.lut[f32_as_u32(xs[e]) >> (32 - kLutBits)];
    uint2 t0[NE], t1[NE];  // {tau[lo], spread[lo]}, {tau[lo+1], spread[lo+1]}
    uint32_t top[NE];      // spread[lo+MC]
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const char* row = pair + off[e];
      t0[e] = *reinterpret_cast<const uint2*>(row);
      if constexpr (MC == 2) t1[e] = *reinterpret_cast<const uint2*>(row + 8);
      top[e] = *reinterpret_cast<const uint32_t*>(row + 8 * MC + 4);
    }
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const float x = xs[e];
      if constexpr (MC == 1) {
        sp[e][0] = (x > u32_as_f32(t0[e].x)) ? top[e] : t0[e].y;
      } else {  // tau[lo] <= tau[lo+1]
        const uint32_t s01 = (x > u32_as_f32(t0[e].x)) ? t1[e].y : t0[e].y;
        sp[e][0] = (x > u32_as_f32(t1[e].x)) ? top[e] : s01;
      }
      accumulate_elem<K>(x, sp[e], a32, sx32);
    }
  } else {
#pragma unroll
    for (int e = 0; e < NE; ++e) encode_elem<K>(tb, xs[e], MC == 1 ? 1 : maxcnt, sp[e], a32, sx32);
  }
}

// End of an item: bit counts from the finished plane bytes, payload store, float32 partial
// sums (at most 8*VEC terms) folded into the thread's float64 sums.
template <int K, int VEC>
__device__ __forceinline__ void finish_item(const uint32_t (&acc)[VEC][(K + 3) / 4], const float (&h32)[K], float sx32,
                                            uint8_t* __restrict__ dst, EncodeStats<K>& st) {
  constexpr int NDW = (VEC * K + 3) / 4;
  constexpr int CW = (VEC + 3) / 4;
  uint32_t pw[K][CW];  // plane bytes of all VEC columns, plane-major
#pragma unroll
  for (int p = 0; p < K; ++p) {
#pragma unroll
    for (int w = 0; w < CW; ++w) pw[p][w] = 0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) pw[p][c / 4] |= ((acc[c][p / 4] >> (8 * (p % 4))) & 0xFFu) << (8 * (c % 4));
  }
  {
    int pi = 0;
#pragma unroll
    for (int p = 0; p < K; ++p) {
#pragma unroll
      for (int w = 0; w < CW; ++w) st.cnt[p] += __popc(pw[p][w]);
#pragma unroll
      for (int q = p + 1; q < K; ++q) {
#pragma unroll
        for (int w = 0; w < CW; ++w) st.dis[pi] += __popc(pw[p][w] ^ pw[q][w]);
        ++pi;
      }
    }
  }
  // payload: byte ((g*m + j)*K + p); the item's VEC*K bytes are contiguous
  if constexpr (VEC > 1) {
    uint32_t out[NDW];
    if constexpr (K == 4) {
#pragma unroll
      for (int c = 0; c < VEC; ++c) out[c] = acc[c][0];
    } else {
#pragma unroll
      for (int w = 0; w < NDW; ++w) out[w] = 0;
#pragma unroll
      for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int p = 0; p < K; ++p) {
          const int b = c * K + p;
          out[b / 4] |= ((acc[c][p / 4] >> (8 * (p % 4))) & 0xFFu) << (8 * (b % 4));
        }
    }
    store_dwords<NDW>(reinterpret_cast<uint32_t*>(dst), out);
  } else {
#pragma unroll
    for (int p = 0; p < K; ++p) dst[p] = uint8_t(acc[0][p / 4] >> (8 * (p % 4)));
  }
  st.Sx += double(sx32);
#pragma unroll
  for (int p = 0; p < K; ++p) st.H[p] += double(h32[p]);
}

// One row's share of an item as it comes from memory: VEC elements in a 16-byte vector, or a
// single element's bits.  Rows are kept in this form while they wait and widened to float32
// only when they are used, so that a load's result is not needed before then.
template <int VEC>
struct RawRow {
  uint4 v;
};
template <>
struct RawRow<1> {
  uint32_t v;
};
template <typename T, int VEC>
__device__ __forceinline__ RawRow<VEC> load_raw(const T* p) {
  RawRow<VEC> r;
  if constexpr (VEC > 1) {
    r.v = load16_stream(p);  // every element of x is read once
  } else if constexpr (sizeof(T) == 4) {
    r.v = f32_as_u32(*reinterpret_cast<const float*>(p));
  } else {
    r.v = uint32_t(*reinterpret_cast<const uint16_t*>(p)) << 16;
  }
  return r;
}
template <int VEC>
__device__ __forceinline__ void widen_raw(const RawRow<VEC>& r, float (&f)[VEC]) {
  if constexpr (VEC > 1) {
    widen(r.v, f);
  } else {
    f[0] = u32_as_f32(r.v);
  }
}

// Plain (not pipelined) item of one column: any number of valid rows.
template <typename T, int K, int MC>
__device__ __forceinline__ void encode_column(const EncodeTables<K>& tb, const T* __restrict__ x,
                                              uint8_t* __restrict__ payload, int64_t n, int64_t m, int64_t g,
                                              int64_t j, int maxcnt, EncodeStats<K>& st) {
  constexpr int NW = (K + 3) / 4;
  const int64_t row0 = g * 8;
  const int nrows = (n - row0) < 8 ? int(n - row0) : 8;
  const T* xc = x + row0 * m + j;
  float xs[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {  // all row loads first, so that they overlap
    RawRow<1> raw;
    raw.v = 0u;
    if (r < nrows) raw = load_raw<T, 1>(xc + r * m);
    float one[1];
    widen_raw<1>(raw, one);
    xs[r] = one[0];  // a missing row reads as +0: it adds nothing to the sums
  }
  float h32[K];
  float sx32 = 0.0f;
#pragma unroll
  for (int p = 0; p < K; ++p) h32[p] = 0.0f;
  uint32_t sp[8][NW];
  encode_group<K, MC, 8>(tb, xs, maxcnt, sp, h32, sx32);
  // M3: row r of the group lands at bit 7-r of each plane byte; missing rows give 0 bits
  uint32_t acc[1][NW];
#pragma unroll
  for (int w = 0; w < NW; ++w) acc[0][w] = 0;
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int w = 0; w < NW; ++w) acc[0][w] = (acc[0][w] << 1) | (r < nrows ? sp[r][w] : 0u);
  finish_item<K, 1>(acc, h32, sx32, payload + ((g * m + j) * K), st);
}

// The pipelined loop over whole rounds of the grid (every thread has an item in every round).
template <typename T, int K, int VEC, int MC>
__device__ __forceinline__ void encode_rounds(const EncodeTables<K>& tb, const T* __restrict__ x,
                                              uint8_t* __restrict__ payload, int64_t m, int64_t ipg, int64_t rounds,
                                              ItemPos pos, const ItemStep& step, RawRow<VEC> (&fr)[8],
                                              EncodeStats<K>& st) {
  constexpr int NW = (K + 3) / 4;
  constexpr int GR = VEC >= ACCEPT_ENCODE_GROUP ? 1 : ACCEPT_ENCODE_GROUP / VEC;  // rows handled together
  // The first item's rows have had the whole table build to arrive.  Waiting for them here
  // (vmcnt 0, the other counters untouched) gives the loop an empty set of outstanding loads
  // on entry whatever code precedes it, so that the waits the compiler places inside the loop
  // are the ones its own steady state needs and no more.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  for (int64_t rd = 0; rd < rounds; ++rd) {
    ItemPos npos = pos;
    item_advance(npos, step, ipg);
    // In the last round there is no next item: every lane then re-reads the first item of the
    // tensor (valid, one cache line per row for the whole wavefront), so that the loads stay
    // unconditional and the compiler can reuse the row registers in place.
    if (rd + 1 >= rounds) { npos.g = 0; npos.jv = 0; }
    const T* nxc = x + npos.g * 8 * m + npos.jv * VEC;
    uint32_t acc[VEC][NW];
    float h32[K];
    float sx32 = 0.0f;
#pragma unroll
    for (int p = 0; p < K; ++p) h32[p] = 0.0f;
#pragma unroll
    for (int c = 0; c < VEC; ++c)
#pragma unroll
      for (int w = 0; w < NW; ++w) acc[c][w] = 0;
#pragma unroll
    for (int r0 = 0; r0 < 8; r0 += GR) {
      float xs[GR * VEC];
#pragma unroll
      for (int rr = 0; rr < GR; ++rr) {
        float row[VEC];
        widen_raw<VEC>(fr[r0 + rr], row);
#pragma unroll
        for (int c = 0; c < VEC; ++c) xs[rr * VEC + c] = row[c];
      }
      uint32_t sp[GR * VEC][NW];
      encode_group<K, MC, GR * VEC>(tb, xs, MC, sp, h32, sx32);
      // M3: row r of the group lands at bit 7-r of each plane byte
#pragma unroll
      for (int rr = 0; rr < GR; ++rr)
#pragma unroll
        for (int c = 0; c < VEC; ++c)
#pragma unroll
          for (int w = 0; w < NW; ++w) acc[c][w] = (acc[c][w] << 1) | sp[rr * VEC + c][w];
#pragma unroll
      for (int rr = 0; rr < GR; ++rr) fr[r0 + rr] = load_raw<T, VEC>(nxc + (r0 + rr) * m);
      // keep the instruction scheduler from mixing groups: it would otherwise hoist the table
      // reads of all 8*VEC elements and run out of registers
      __builtin_amdgcn_sched_barrier(0);
    }
    finish_item<K, VEC>(acc, h32, sx32, payload + ((pos.g * m + pos.jv * VEC) * K), st);
    pos = npos;
  }
}

// Fused M1..M4.  Items whose eight rows all exist run through a software-pipelined loop:
// row r of the next item is requested as soon as row r of the current item has been
// consumed, so a wavefront always has loads in flight while it works; the first item's rows
// are requested before the tables are built.  The last, partial row group (n % 8 != 0) and
// the rare case of more than two thresholds per bucket take the plain path.
template <typename T, int K, int VEC>
__global__ __launch_bounds__(kBlock, ACCEPT_ENCODE_WAVES) void mbq_encode_kernel(const T* __restrict__ x,
                                                             const float* __restrict__ alpha_prev,
                                                             uint8_t* __restrict__ payload,
                                                             double* __restrict__ partials, int64_t n, int64_t m,
                                                             int64_t ipg, ItemStep step) {
  constexpr int NPAIR = K * (K - 1) / 2;
  constexpr int NSTAT = nstat_of(K);
  __shared__ EncodeTables<K> tb;
  __shared__ StatScratch red;

  const int tid = threadIdx.x;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t items_full = (n / 8) * ipg;  // items of complete row groups come first
  int64_t it = int64_t(blockIdx.x) * kBlock + tid;
  ItemPos pos;
  pos.g = it / ipg;
  pos.jv = it - pos.g * ipg;

  // Whole rounds (every thread of the grid has an item) go through the pipelined loop; what is
  // left of the complete row groups is then spread over the grid one column at a time, so that
  // no thread carries a whole extra item while the others idle.
  const int64_t rounds = items_full / stride;
  RawRow<VEC> fr[8];
  if (rounds > 0) {
    const T* xc = x + pos.g * 8 * m + pos.jv * VEC;
#pragma unroll
    for (int r = 0; r < 8; ++r) fr[r] = load_raw<T, VEC>(xc + r * m);
  }

  build_encode_tables<K>(alpha_prev, tb);
  // the same value in every lane: read it into a scalar register, so that the choice of path
  // below is a scalar branch and not a divergent one whose sides run one after the other
  const int maxcnt = __builtin_amdgcn_readfirstlane(tb.maxcnt);

  EncodeStats<K> st;
  st.Sx = 0.0;
#pragma unroll
  for (int p = 0; p < K; ++p) { st.H[p] = 0.0; st.cnt[p] = 0; }
#pragma unroll
  for (int i = 0; i < (NPAIR > 0 ? NPAIR : 1); ++i) st.dis[i] = 0;

  const int64_t gtid = int64_t(blockIdx.x) * kBlock + tid;
  // whole rounds pipelined, then the items of the last, incomplete round one column per thread
  const int64_t first_left = rounds * stride;
  const int64_t cols_left = (items_full - first_left) * VEC;
  if (maxcnt == 1) {
    encode_rounds<T, K, VEC, 1>(tb, x, payload, m, ipg, rounds, pos, step, fr, st);
    for (int64_t s = gtid; s < cols_left; s += stride) {
      const int64_t item = first_left + s / VEC;
      const int64_t g = item / ipg;
      encode_column<T, K, 1>(tb, x, payload, n, m, g, (item - g * ipg) * VEC + s % VEC, 1, st);
    }
  } else if (maxcnt == 2 && K <= 4) {
    encode_rounds<T, K, VEC, 2>(tb, x, payload, m, ipg, rounds, pos, step, fr, st);
    for (int64_t s = gtid; s < cols_left; s += stride) {
      const int64_t item = first_left + s / VEC;
      const int64_t g = item / ipg;
      encode_column<T, K, 2>(tb, x, payload, n, m, g, (item - g * ipg) * VEC + s % VEC, 2, st);
    }
  } else {
    // several thresholds share a bucket (levels closer than a bucket's width): rare.  One column
    // per thread keeps this path's register needs out of the kernel's budget.
    const int64_t cols_full = (n / 8) * m;
    for (int64_t s = gtid; s < cols_full; s += stride) {
      const int64_t g = s / m;
      encode_column<T, K, 0>(tb, x, payload, n, m, g, s - g * m, maxcnt, st);
    }
  }
  // the last, partial row group (n % 8 != 0), one column per thread
  if (n % 8 != 0) {
    for (int64_t j = gtid; j < m; j += stride)
      encode_column<T, K, 0>(tb, x, payload, n, m, n / 8, j, maxcnt, st);
  }

  // M4: workgroup totals in a fixed order -> one record per workgroup, stat-major
  double sv[NSTAT];
#pragma unroll
  for (int p = 0; p < K; ++p) sv[p] = st.H[p];
  sv[K] = st.Sx;
#pragma unroll
  for (int p = 0; p < K; ++p) sv[K + 1 + p] = double(st.cnt[p]);
#pragma unroll
  for (int i = 0; i < NPAIR; ++i) sv[2 * K + 1 + i] = double(st.dis[i]);
  const double total = block_sum_stats<NSTAT>(sv, red);
  if (tid < NSTAT) partials[int64_t(tid) * gridDim.x + blockIdx.x] = total;
}

// ========================================================================= finalize (M5)
// One workgroup: fixed-order float64 totals (one wavefront per statistic), then one thread
// solves alpha_cur = (B^T B)^-1 B^T x by Gaussian elimination with row pivoting, applies the
// moving average with beta = min(0.9, (1+t)/(10+t)) and m_q = mean(B alpha_t - x);
// header = [alpha_t, m_q].  K is a template parameter so that the k x k system lives in
// registers.
constexpr int kFinBlock = kBlock;
constexpr int kFinRPT = (kEncodeGridMax + kFinBlock - 1) / kFinBlock;  // records per thread, at most
template <int K>
__global__ __launch_bounds__(kFinBlock) void mbq_finalize_kernel(const double* __restrict__ partials, int nrec,
                                                               const float* __restrict__ alpha_prev, double n_elems,
                                                               double t, float* __restrict__ header) {
  constexpr int NSTAT = nstat_of(K);
  __shared__ double tot[NSTAT];
  const int tid = threadIdx.x;
  // every thread takes records tid, tid+256, ... (at most kFinRPT) of every statistic; the loads
  // of a statistic are all issued before their adds, so few memory latencies are paid.  Then
  // the fixed-order workgroup sum: the totals do not depend on timing.
  __shared__ StatScratch red;
  double a[NSTAT];
  double v[NSTAT][kFinRPT];
#pragma unroll
  for (int s = 0; s < NSTAT; ++s)
#pragma unroll
    for (int i = 0; i < kFinRPT; ++i) {
      const int b = tid + i * kFinBlock;
      v[s][i] = (b < nrec) ? partials[int64_t(s) * nrec + b] : 0.0;
    }
#pragma unroll
  for (int s = 0; s < NSTAT; ++s) {
    a[s] = v[s][0];
#pragma unroll
    for (int i = 1; i < kFinRPT; ++i) a[s] += v[s][i];
  }
  const double total = block_sum_stats<NSTAT>(a, red);
  if (tid < NSTAT) tot[tid] = total;
  __syncthreads();
  if (tid != 0) return;
  double G[K][K], b[K], Sb[K], a_prev[K], cur[K];
  const double Sx = tot[K];
  {
    int pi = 0;
#pragma unroll
    for (int p = 0; p < K; ++p) {
      a_prev[p] = double(alpha_prev[p]);
      b[p] = 2.0 * tot[p] - Sx;                 // B^T x = 2 * (sum over +1 entries) - sum(x)
      Sb[p] = 2.0 * tot[K + 1 + p] - n_elems;   // 1^T B
      G[p][p] = n_elems;
#pragma unroll
      for (int q = p + 1; q < K; ++q) {
        G[p][q] = G[q][p] = n_elems - 2.0 * tot[2 * K + 1 + pi];
        ++pi;
      }
    }
  }
  bool singular = false;
  double inv[K];
#pragma unroll
  for (int col = 0; col < K; ++col) {
    // bring the largest |entry| of the column to the diagonal (compare-and-swap keeps the
    // indices static, so the system stays in registers)
#pragma unroll
    for (int r = col + 1; r < K; ++r) {
      if (fabs(G[r][col]) > fabs(G[col][col])) {
#pragma unroll
        for (int c = 0; c < K; ++c) { const double tmp = G[col][c]; G[col][c] = G[r][c]; G[r][c] = tmp; }
        const double tb_ = b[col]; b[col] = b[r]; b[r] = tb_;
      }
    }
    if (fabs(G[col][col]) < 1e-9 * n_elems) singular = true;
    inv[col] = 1.0 / G[col][col];  // one division per column; its products differ from quotients by an ulp
    if (!singular) {
#pragma unroll
      for (int r = col + 1; r < K; ++r) {
        const double fct = G[r][col] * inv[col];
#pragma unroll
        for (int c = col; c < K; ++c) G[r][c] -= fct * G[col][c];
        b[r] -= fct * b[col];
      }
    }
  }
#pragma unroll
  for (int r = K - 1; r >= 0; --r) {
    double acc = b[r];
#pragma unroll
    for (int c = r + 1; c < K; ++c) acc -= G[r][c] * cur[c];
    cur[r] = singular ? a_prev[r] : acc * inv[r];
  }
  double beta = (1.0 + t) / (10.0 + t);
  if (beta > 0.9) beta = 0.9;
  double dot = 0.0;
#pragma unroll
  for (int p = 0; p < K; ++p) {
    const float a_t = float(beta * a_prev[p] + (1.0 - beta) * (singular ? a_prev[p] : cur[p]));
    header[p] = a_t;
    dot += double(a_t) * Sb[p];
  }
  header[K] = float((dot - Sx) / n_elems);
}

// ================================================ comparison layout: one byte per binary base
// ACCEPT_LAYOUT_UNENCODED: B itself, +1 / -1 as bytes, element-major with the k bases
// innermost ("w/o enc." in the paper's size table).  Same levels, same sums and the same
// finalize kernel as the bit-plane path; plain flat loops, four elements per thread and step.
template <typename T, int K>
__global__ __launch_bounds__(kBlock) void mbq_encode_plain_kernel(const T* __restrict__ x,
                                                                  const float* __restrict__ alpha_prev,
                                                                  uint8_t* __restrict__ payload,
                                                                  double* __restrict__ partials, int64_t N) {
  constexpr int NW = (K + 3) / 4;
  constexpr int NPAIR = K * (K - 1) / 2;
  constexpr int NSTAT = nstat_of(K);
  __shared__ EncodeTables<K> tb;
  __shared__ StatScratch red;
  const int tid = threadIdx.x;
  build_encode_tables<K>(alpha_prev, tb);
  const int maxcnt = __builtin_amdgcn_readfirstlane(tb.maxcnt);
  EncodeStats<K> st;
  st.Sx = 0.0;
#pragma unroll
  for (int p = 0; p < K; ++p) { st.H[p] = 0.0; st.cnt[p] = 0; }
#pragma unroll
  for (int i = 0; i < (NPAIR > 0 ? NPAIR : 1); ++i) st.dis[i] = 0;

  // one element: level, sums, and its k bytes (+1 -> 0x01, -1 -> 0xFF) into bytes[0..K)
  auto element = [&](float v, uint8_t (&bytes)[K], float (&h32)[K], float& sx32) {
    uint32_t sp[NW];
    encode_elem<K>(tb, v, maxcnt, sp, h32, sx32);
    uint32_t bit[K];
#pragma unroll
    for (int p = 0; p < K; ++p) {
      bit[p] = (sp[p / 4] >> (8 * (p % 4))) & 1u;
      bytes[p] = bit[p] ? uint8_t(0x01) : uint8_t(0xFF);
      st.cnt[p] += bit[p];
    }
    int pi = 0;
#pragma unroll
    for (int p = 0; p < K; ++p)
#pragma unroll
      for (int q = p + 1; q < K; ++q) st.dis[pi++] += bit[p] ^ bit[q];
  };

  const int64_t quads = N / 4;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kBlock + tid;
  for (int64_t u = gtid; u < quads; u += stride) {
    float f[4];
    load_quad<T>(x + 4 * u, f);
    float h32[K];
    float sx32 = 0.0f;
#pragma unroll
    for (int p = 0; p < K; ++p) h32[p] = 0.0f;
    uint32_t out[K];  // 4 elements x K bytes = K dwords
#pragma unroll
    for (int w = 0; w < K; ++w) out[w] = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      uint8_t bytes[K];
      element(f[e], bytes, h32, sx32);
#pragma unroll
      for (int p = 0; p < K; ++p) {
        const int b = e * K + p;
        out[b / 4] |= uint32_t(bytes[p]) << (8 * (b % 4));
      }
    }
    store_dwords<K>(reinterpret_cast<uint32_t*>(payload) + u * K, out);
    st.Sx += double(sx32);
#pragma unroll
    for (int p = 0; p < K; ++p) st.H[p] += double(h32[p]);
  }
  {
    const int64_t i = quads * 4 + gtid;
    if (i < N) {
      float h32[K];
      float sx32 = 0.0f;
#pragma unroll
      for (int p = 0; p < K; ++p) h32[p] = 0.0f;
      uint8_t bytes[K];
      element(load_one(x + i), bytes, h32, sx32);
#pragma unroll
      for (int p = 0; p < K; ++p) payload[i * K + p] = bytes[p];
      st.Sx += double(sx32);
#pragma unroll
      for (int p = 0; p < K; ++p) st.H[p] += double(h32[p]);
    }
  }
  double sv[NSTAT];
#pragma unroll
  for (int p = 0; p < K; ++p) sv[p] = st.H[p];
  sv[K] = st.Sx;
#pragma unroll
  for (int p = 0; p < K; ++p) sv[K + 1 + p] = double(st.cnt[p]);
#pragma unroll
  for (int i = 0; i < NPAIR; ++i) sv[2 * K + 1 + i] = double(st.dis[i]);
  const double total = block_sum_stats<NSTAT>(sv, red);
  if (tid < NSTAT) partials[int64_t(tid) * gridDim.x + blockIdx.x] = total;
}

template <typename TO, int K>
__global__ __launch_bounds__(kBlock) void mbq_decode_plain_kernel(const uint8_t* __restrict__ payload,
                                                                  const float* __restrict__ header,
                                                                  TO* __restrict__ xhat, int64_t N) {
  constexpr int P = 1 << K;
  __shared__ float lut[P];
  const int tid = threadIdx.x;
  if (tid < P) {
    float v = 0.0f;
#pragma unroll
    for (int p = 0; p < K; ++p) {
      const float a = header[p];
      v = __fadd_rn(v, ((tid >> p) & 1) ? a : -a);
    }
    lut[tid] = __fsub_rn(v, header[K]);
  }
  __syncthreads();
  const int64_t quads = N / 4;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kBlock + tid;
  for (int64_t u = gtid; u < quads; u += stride) {
    uint32_t w[K];
#pragma unroll
    for (int i = 0; i < K; ++i) w[i] = reinterpret_cast<const uint32_t*>(payload)[u * K + i];
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      uint32_t pat = 0;
#pragma unroll
      for (int p = 0; p < K; ++p) {
        const int b = e * K + p;
        const uint32_t byte = (w[b / 4] >> (8 * (b % 4))) & 0xFFu;
        pat |= (((byte >> 7) & 1u) ^ 1u) << p;  // +1 (0x01) -> bit 1, -1 (0xFF) -> bit 0
      }
      f[e] = lut[pat];
    }
    store_quad<TO>(xhat + 4 * u, f);
  }
  const int64_t i = quads * 4 + gtid;
  if (i < N) {
    uint32_t pat = 0;
#pragma unroll
    for (int p = 0; p < K; ++p) pat |= (((uint32_t(payload[i * K + p]) >> 7) & 1u) ^ 1u) << p;
    store_one(xhat + i, lut[pat]);
  }
}

// ====================================================================== decode (D1 + D2)
template <typename TO, int K, int VEC>
__global__ __launch_bounds__(kBlock) void mbq_decode_kernel(const uint8_t* __restrict__ payload,
                                                             const float* __restrict__ header,
                                                             TO* __restrict__ xhat, int64_t n, int64_t m,
                                                             int64_t ipg, int64_t items, ItemStep step) {
  constexpr int P = 1 << K;
  constexpr int NDW = (VEC * K + 3) / 4;
  __shared__ float lut[P];
  const int tid = threadIdx.x;
  if (tid < P) {
    // x_hat of a sign pattern: float32 sum of +-alpha_p, p = 0..k-1 from 0, minus m_q
    float v = 0.0f;
#pragma unroll
    for (int p = 0; p < K; ++p) {
      const float a = header[p];
      v = __fadd_rn(v, ((tid >> p) & 1) ? a : -a);
    }
    lut[tid] = __fsub_rn(v, header[K]);
  }
  __syncthreads();

  int64_t it = int64_t(blockIdx.x) * kBlock + tid;
  ItemPos pos;
  pos.g = it / ipg;
  pos.jv = it - pos.g * ipg;
  for (; it < items; it += int64_t(gridDim.x) * kBlock, item_advance(pos, step, ipg)) {
    const uint8_t* src = payload + ((pos.g * m + pos.jv * VEC) * K);
    uint32_t w[NDW];
    if constexpr (VEC > 1) {
      const Dwords<NDW> in = *reinterpret_cast<const Dwords<NDW>*>(src);
#pragma unroll
      for (int i = 0; i < NDW; ++i) w[i] = in.v[i];
    } else {
#pragma unroll
      for (int i = 0; i < NDW; ++i) w[i] = 0;
#pragma unroll
      for (int p = 0; p < K; ++p) w[p / 4] |= uint32_t(src[p]) << (8 * (p % 4));
    }
    const int64_t row0 = pos.g * 8;
    TO* dst = xhat + pos.jv * VEC;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      if (row0 + r < n) {
        float f[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
          uint32_t pat = 0;
#pragma unroll
          for (int p = 0; p < K; ++p) {
            const int b = c * K + p;
            pat |= ((w[b / 4] >> (8 * (b % 4) + 7 - r)) & 1u) << p;
          }
          f[c] = lut[pat];
        }
        if constexpr (VEC > 1) {
          store_vec(dst + (row0 + r) * m, f);
        } else {
          store_one(dst + (row0 + r) * m, f[0]);
        }
      }
    }
  }
}

// ======================================================= residue initialisation of alpha
// Pass j: sum of |rho_j| with rho_0 = x, rho_(i+1) = rho_i - alpha_i sign(rho_i), sign(0) = +1,
// carried in float64; alpha_0..alpha_(j-1) are read from device memory.
template <typename T>
__global__ __launch_bounds__(kBlock) void mbq_init_pass_kernel(const T* __restrict__ x, int64_t N, int j,
                                                                const float* __restrict__ alpha,
                                                                double* __restrict__ partials) {
  __shared__ double red[kBlock / kWave];
  double a[8];
  for (int i = 0; i < j; ++i) a[i] = double(alpha[i]);
  double acc = 0.0;
  for (int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x; i < N; i += int64_t(gridDim.x) * kBlock) {
    double rho = double(load_one(x + i));
    for (int q = 0; q < j; ++q) rho -= (rho >= 0.0) ? a[q] : -a[q];
    acc += fabs(rho);
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = red[0];
    for (int w = 1; w < kBlock / kWave; ++w) t += red[w];
    partials[blockIdx.x] = t;
  }
}
__global__ __launch_bounds__(kBlock) void mbq_init_finalize_kernel(const double* __restrict__ partials, int nrec,
                                                                    double n_elems, int j, float* __restrict__ alpha) {
  __shared__ double red[kBlock];
  const int tid = threadIdx.x;
  double a = 0.0;
  for (int b = tid; b < nrec; b += kBlock) a += partials[b];
  red[tid] = a;
  __syncthreads();
  for (int off = kBlock / 2; off > 0; off >>= 1) {
    if (tid < off) red[tid] += red[tid + off];
    __syncthreads();
  }
  if (tid == 0) alpha[j] = float(red[0] / n_elems);
}

// ============================================================================= host side
int vec_for(int dtype, int64_t m) {
  const int v = dtype == ACCEPT_BF16 ? 8 : 4;
  return (m % v == 0) ? v : 1;
}

int grid_for(int64_t items, int grid_max) {
  int64_t blocks = (items + kBlock - 1) / kBlock;
  if (blocks < 1) blocks = 1;
  return int(blocks < grid_max ? blocks : grid_max);
}

ItemStep step_for(int grid, int64_t ipg) {
  const int64_t stride = int64_t(grid) * kBlock;
  ItemStep st;
  st.dg = stride / ipg;
  st.dj = stride % ipg;
  return st;
}

template <typename T, int K, int VEC>
hipError_t launch_encode(const accept_desc& d, const MPlan& p, const T* x, const float* alpha_prev, uint8_t* payload,
                         double* partials, hipStream_t s) {
  const int64_t ipg = d.m / VEC;
  hipLaunchKernelGGL((mbq_encode_kernel<T, K, VEC>), dim3(p.grid), dim3(kBlock), 0, s, x, alpha_prev, payload,
                     partials, d.n, d.m, ipg, step_for(p.grid, ipg));
  return hipGetLastError();
}

template <typename T, int VEC>
hipError_t encode_k(const accept_desc& d, const MPlan& p, const T* x, const float* alpha_prev, uint8_t* payload,
                    double* partials, hipStream_t s) {
  switch (d.bits) {
    case 1: return launch_encode<T, 1, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 2: return launch_encode<T, 2, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 3: return launch_encode<T, 3, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 4: return launch_encode<T, 4, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 5: return launch_encode<T, 5, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 6: return launch_encode<T, 6, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 7: return launch_encode<T, 7, VEC>(d, p, x, alpha_prev, payload, partials, s);
    case 8: return launch_encode<T, 8, VEC>(d, p, x, alpha_prev, payload, partials, s);
    default: return hipErrorInvalidValue;
  }
}

template <typename TO, int K, int VEC>
hipError_t launch_decode(const accept_desc& d, const uint8_t* payload, const float* header, TO* xhat, hipStream_t s) {
  const int64_t ipg = d.m / VEC;
  const int64_t items = ((d.n + 7) / 8) * ipg;
  const int grid = grid_for(items, kDecodeGridMax);
  hipLaunchKernelGGL((mbq_decode_kernel<TO, K, VEC>), dim3(grid), dim3(kBlock), 0, s, payload, header, xhat, d.n,
                     d.m, ipg, items, step_for(grid, ipg));
  return hipGetLastError();
}

template <typename TO, int VEC>
hipError_t decode_k(const accept_desc& d, const uint8_t* payload, const float* header, TO* xhat, hipStream_t s) {
  switch (d.bits) {
    case 1: return launch_decode<TO, 1, VEC>(d, payload, header, xhat, s);
    case 2: return launch_decode<TO, 2, VEC>(d, payload, header, xhat, s);
    case 3: return launch_decode<TO, 3, VEC>(d, payload, header, xhat, s);
    case 4: return launch_decode<TO, 4, VEC>(d, payload, header, xhat, s);
    case 5: return launch_decode<TO, 5, VEC>(d, payload, header, xhat, s);
    case 6: return launch_decode<TO, 6, VEC>(d, payload, header, xhat, s);
    case 7: return launch_decode<TO, 7, VEC>(d, payload, header, xhat, s);
    case 8: return launch_decode<TO, 8, VEC>(d, payload, header, xhat, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

MPlan make_mplan(const accept_desc& d) {
  MPlan p{};
  p.vec = vec_for(d.in_dtype, d.m);
  p.G = (d.n + 7) / 8;
  p.items = p.G * (d.m / p.vec);
  // Grid of the encode kernel.  Its fast loop runs whole rounds (every thread of the grid has an
  // item) and what is left over goes one column per thread, so a tensor with fewer items than
  // the largest grid has threads gets the largest grid that still fills one round (rounding the
  // grid up instead would leave every item to the slower leftover path).  The columns of a last,
  // partial row group also go one per thread: the grid is at least wide enough for them.
  {
    const int64_t items_full = (d.n / 8) * (d.m / p.vec);
    int64_t blocks = items_full / kBlock;
    const int64_t tail_blocks = (d.n % 8 != 0) ? (d.m + kBlock - 1) / kBlock : 0;
    if (blocks < tail_blocks) blocks = tail_blocks;
    if (blocks < 1) blocks = 1;
    p.grid = int(blocks < kEncodeGridMax ? blocks : kEncodeGridMax);
  }
  p.nstat = nstat_of(d.bits);
  // records of the encode kernel (stat-major, kEncodeGridMax wide at most) and, for the
  // residue initialisation, kInitGrid partial sums: both fit the same area
  size_t bytes = size_t(nstat_of(8)) * 2048 * sizeof(double);
  p.bytes = (bytes + 255) / 256 * 256;
  return p;
}

template <typename T>
hipError_t encode_plain_k(const accept_desc& d, int grid, const T* x, const float* alpha_prev, uint8_t* payload,
                          double* partials, hipStream_t s) {
  const int64_t N = d.n * d.m;
#define ACCEPT_ENC(KK)                                                                                          \
  case KK:                                                                                                      \
    hipLaunchKernelGGL((mbq_encode_plain_kernel<T, KK>), dim3(grid), dim3(kBlock), 0, s, x, alpha_prev, payload, \
                       partials, N);                                                                            \
    break;
  switch (d.bits) {
    ACCEPT_ENC(1) ACCEPT_ENC(2) ACCEPT_ENC(3) ACCEPT_ENC(4) ACCEPT_ENC(5) ACCEPT_ENC(6) ACCEPT_ENC(7) ACCEPT_ENC(8)
    default: return hipErrorInvalidValue;
  }
#undef ACCEPT_ENC
  return hipGetLastError();
}

template <typename TO>
hipError_t decode_plain_k(const accept_desc& d, const uint8_t* payload, const float* header, TO* xhat,
                          hipStream_t s) {
  const int64_t N = d.n * d.m;
  const int grid = grid_for(N / 4 + 4, kDecodeGridMax);
#define ACCEPT_DEC(KK)                                                                                       \
  case KK:                                                                                                   \
    hipLaunchKernelGGL((mbq_decode_plain_kernel<TO, KK>), dim3(grid), dim3(kBlock), 0, s, payload, header, \
                       xhat, N);                                                                             \
    break;
  switch (d.bits) {
    ACCEPT_DEC(1) ACCEPT_DEC(2) ACCEPT_DEC(3) ACCEPT_DEC(4) ACCEPT_DEC(5) ACCEPT_DEC(6) ACCEPT_DEC(7) ACCEPT_DEC(8)
    default: return hipErrorInvalidValue;
  }
#undef ACCEPT_DEC
  return hipGetLastError();
}

hipError_t launch_mbq_compress(const accept_desc& d, const MPlan& p, const void* x, const float* alpha_prev,
                               void* header, void* payload, void* ws, hipStream_t s, StageTimer* tm) {
  double* partials = static_cast<double*>(ws);
  uint8_t* pl = static_cast<uint8_t*>(payload);
  hipError_t e;
  mark(tm, s);
  int nrec = p.grid;
  if (d.layout == ACCEPT_LAYOUT_UNENCODED) {
    nrec = grid_for(d.n * d.m / 4 + 4, kEncodeGridMax);
    e = d.in_dtype == ACCEPT_BF16
            ? encode_plain_k<bf16_t>(d, nrec, static_cast<const bf16_t*>(x), alpha_prev, pl, partials, s)
            : encode_plain_k<float>(d, nrec, static_cast<const float*>(x), alpha_prev, pl, partials, s);
  } else if (d.in_dtype == ACCEPT_BF16) {
    const bf16_t* xb = static_cast<const bf16_t*>(x);
    e = p.vec == 8 ? encode_k<bf16_t, 8>(d, p, xb, alpha_prev, pl, partials, s)
                   : encode_k<bf16_t, 1>(d, p, xb, alpha_prev, pl, partials, s);
  } else {
    const float* xf = static_cast<const float*>(x);
    e = p.vec == 4 ? encode_k<float, 4>(d, p, xf, alpha_prev, pl, partials, s)
                   : encode_k<float, 1>(d, p, xf, alpha_prev, pl, partials, s);
  }
  if (e != hipSuccess) return e;
  mark(tm, s);
  const double n_elems = double(d.n) * double(d.m);
  float* hdr = static_cast<float*>(header);
#define ACCEPT_FIN(KK)                                                                                         \
  case KK:                                                                                                     \
    hipLaunchKernelGGL(mbq_finalize_kernel<KK>, dim3(1), dim3(kFinBlock), 0, s, partials, nrec, alpha_prev,   \
                       n_elems, double(d.t), hdr);                                                             \
    break;
  switch (d.bits) {
    ACCEPT_FIN(1) ACCEPT_FIN(2) ACCEPT_FIN(3) ACCEPT_FIN(4) ACCEPT_FIN(5) ACCEPT_FIN(6) ACCEPT_FIN(7) ACCEPT_FIN(8)
    default: return hipErrorInvalidValue;
  }
#undef ACCEPT_FIN
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  mark(tm, s);
  return hipSuccess;
}

hipError_t launch_mbq_decompress(const accept_desc& d, const void* header, const void* payload, void* xhat,
                                 hipStream_t s, StageTimer* tm) {
  const uint8_t* pl = static_cast<const uint8_t*>(payload);
  const float* hd = static_cast<const float*>(header);
  const int vec = vec_for(d.out_dtype, d.m);
  hipError_t e;
  mark(tm, s);
  if (d.layout == ACCEPT_LAYOUT_UNENCODED) {
    e = d.out_dtype == ACCEPT_BF16 ? decode_plain_k<bf16_t>(d, pl, hd, static_cast<bf16_t*>(xhat), s)
                                   : decode_plain_k<float>(d, pl, hd, static_cast<float*>(xhat), s);
  } else if (d.out_dtype == ACCEPT_BF16) {
    bf16_t* o = static_cast<bf16_t*>(xhat);
    e = vec == 8 ? decode_k<bf16_t, 8>(d, pl, hd, o, s) : decode_k<bf16_t, 1>(d, pl, hd, o, s);
  } else {
    float* o = static_cast<float*>(xhat);
    e = vec == 4 ? decode_k<float, 4>(d, pl, hd, o, s) : decode_k<float, 1>(d, pl, hd, o, s);
  }
  if (e != hipSuccess) return e;
  mark(tm, s);
  return hipSuccess;
}

hipError_t launch_mbq_init(const accept_desc& d, const MPlan& p, const void* x, float* alpha0, void* ws,
                           hipStream_t s) {
  (void)p;
  double* partials = static_cast<double*>(ws);
  const int64_t N = d.n * d.m;
  const int grid = grid_for(N, kInitGrid);
  for (int j = 0; j < d.bits; ++j) {
    if (d.in_dtype == ACCEPT_BF16)
      hipLaunchKernelGGL((mbq_init_pass_kernel<bf16_t>), dim3(grid), dim3(kBlock), 0, s,
                         static_cast<const bf16_t*>(x), N, j, alpha0, partials);
    else
      hipLaunchKernelGGL((mbq_init_pass_kernel<float>), dim3(grid), dim3(kBlock), 0, s, static_cast<const float*>(x),
                         N, j, alpha0, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mbq_init_finalize_kernel, dim3(1), dim3(kBlock), 0, s, partials, grid, double(N), j, alpha0);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace accept
