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

// Launch shapes.  The bit-plane encoder runs one workgroup of 8 wavefronts per compute unit
// (256 on this chip): the wavefronts of a compute unit share one set of tables in local memory.
// The comparison-layout encoder and the residue pass are plain 256-thread kernels.
constexpr int kEncBlock = 512;
constexpr int kEncWaves = kEncBlock / kWave;
// Wavefronts draw their work from counters in device memory; the workgroups with block indices
// 8i .. 8i+7 (under round-robin dispatch one on each of the chip's eight dies) share counter i.
constexpr int kGroupBlocks = 8;
constexpr int kGroupSlots = 64;     // wave-items a group takes out of every sweep over the tensor
constexpr int kCounterStride = 64;  // uint32 words between two counters (256 bytes: their own cache lines)
constexpr int kEncodeGridMax = 256;
constexpr int kPlainGridMax = 768;
constexpr int kDecodeGridMax = 8192;
constexpr int kInitGrid = 1024;
constexpr int kMaxRecords = 2048;  // per-workgroup records the workspace has room for
constexpr int kMaxWaves = 16;      // wavefronts of the largest workgroup
constexpr int kMaxGroups = kEncodeGridMax / kGroupBlocks;
static_assert(size_t(kMaxGroups) * kCounterStride * sizeof(uint32_t) <= kCtrlBytes, "the control block holds the counters");
static_assert(kEncodeGridMax <= kMaxRecords && kPlainGridMax <= kMaxRecords && kInitGrid <= kMaxRecords, "records");

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
__device__ __forceinline__ void build_levels(const float (&alpha)[K], float* lv_raw, float* lv_sorted,
                                             uint32_t* pat_sorted) {
  constexpr int P = 1 << K;
  const int pat = threadIdx.x;
  float lv = 0.0f;
  if (pat < P) {
#pragma unroll
    for (int j = 0; j < K; ++j) lv = __fadd_rn(lv, ((pat >> j) & 1) ? alpha[j] : -alpha[j]);
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
constexpr int kLutBits = 12;
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


// The bucket table and the largest number of thresholds inside one bucket.
//   lo(b) = #{tau_i < smallest value of bucket b}, through `count_below(value)`;
//   thresholds inside bucket b = lo(value-order successor of b) - lo(b).  The successor is b+1 on
//   the positive side (b < kLutSize/2) and b-1 on the negative side, where bucket kLutSize/2 (-0)
//   is followed by bucket 0.  Buckets of NaN bit patterns give differences <= 0: ignored.
// A thread takes CH = 8 consecutive buckets (two dwords of the table; never across the sign
// boundary).  lo is monotone along a side, and with a few thresholds among 4096 buckets almost
// every chunk has the same lo at both ends: then every bucket of it has that lo and no threshold
// inside, and only the step to the chunk's successor bucket is left to look at.  The few chunks
// with a threshold inside are then redone one after the other by the whole wavefront, lane j
// taking bucket j of the chunk (one evaluation per chunk instead of eight in a row by one lane).
template <int SHIFT, typename F>
__device__ __forceinline__ int build_bucket_table(uint8_t* lut, F count_below) {
  constexpr int CH = 8;
  static_assert(kLutSize % (2 * CH) == 0, "chunks stay on one side of the sign boundary");
  static_assert((kLutSize / CH) % kWave == 0, "all lanes of a wavefront run the same number of rounds");
  uint32_t* lut32 = reinterpret_cast<uint32_t*>(lut);
  const int lane = threadIdx.x & (kWave - 1);
  int mymax = 0;
  // Chunk c goes to thread (c * 67) mod 512 of its round: the thresholds sit in a few
  // neighbouring chunks (values of similar magnitude), and this spreads those chunks over the
  // wavefronts instead of leaving them all to one.
  constexpr int NCH = kLutSize / CH;
  static_assert(NCH == 512, "the chunk permutation below is a bijection on 512 chunks");
#pragma nounroll
  for (int slot = threadIdx.x; slot < NCH; slot += blockDim.x) {
    const int b0 = ((slot * 67) & (NCH - 1)) * CH;
    const bool neg = b0 >= kLutSize / 2;
    // the chunk's first and last bucket in value order, and the bucket that follows the last
    const int b_first = neg ? b0 + CH - 1 : b0;
    const int b_last = neg ? b0 : b0 + CH - 1;
    int b_succ = neg ? b0 - 1 : b0 + CH;
    if (neg && b0 == kLutSize / 2) b_succ = 0;                  // -0's bucket is followed by +0's
    const bool has_succ = neg || b0 + CH < kLutSize / 2;        // the top positive buckets hold NaN patterns
    const int lo_first = count_below(bucket_vmin(b_first));
    const int lo_last = count_below(bucket_vmin(b_last));
    const int lo_succ = has_succ ? count_below(bucket_vmin(b_succ)) : lo_last;
    const bool steps_inside = lo_first != lo_last;
    if (!steps_inside) {
      const int cnt = lo_succ - lo_last;
      mymax = cnt > mymax ? cnt : mymax;
    }
    const uint32_t fill = (uint32_t(lo_first) * 0x01010101u) << SHIFT;  // lo < 32 when shifted by 3: no carry between bytes
    lut32[b0 / 4] = fill;
    lut32[b0 / 4 + 1] = fill;
    // chunks with a threshold inside (their entries were just filled with a placeholder)
    uint64_t pending = __ballot(steps_inside);
    while (pending != 0) {  // the same in every lane
      const int src = __ffsll((unsigned long long)pending) - 1;
      pending &= pending - 1;
      const int cb0 = __builtin_amdgcn_readlane(b0, src);
      const int c_succ = __builtin_amdgcn_readlane(lo_succ, src);
      const bool cneg = cb0 >= kLutSize / 2;
      const int j = lane & (CH - 1);  // lanes 8.. repeat the work of lanes 0..7 (and store the same bytes)
      const int lo_j = count_below(bucket_vmin(cb0 + j));
      lut[cb0 + j] = uint8_t(uint32_t(lo_j) << SHIFT);
      // thresholds inside bucket cb0 + j: lo of its successor (inside the chunk, else the chunk's) minus its own
      const int lo_up = __shfl(lo_j, (lane & ~(CH - 1)) | ((j + 1) & (CH - 1)), kWave);
      const int lo_down = __shfl(lo_j, (lane & ~(CH - 1)) | ((j + CH - 1) & (CH - 1)), kWave);
      const int next = cneg ? (j > 0 ? lo_down : c_succ) : (j < CH - 1 ? lo_up : c_succ);
      const int cnt = next - lo_j;
      mymax = cnt > mymax ? cnt : mymax;
    }
  }
  return mymax;
}

// M1 and the search tables.  alpha[0..K) = the previous coefficients, already in registers (the
// caller loads them first thing, so that their trip to memory overlaps its other set-up work).
template <int K>
__device__ __forceinline__ void build_encode_tables(const float (&alpha)[K], EncodeTables<K>& tb) {
  using TB = EncodeTables<K>;
  constexpr int P = TB::P;
  const int tid = threadIdx.x;
  const int nthr = blockDim.x;  // at least P = 256 for K = 8
  int mymax = 0;
  if (tid == 0) tb.maxcnt = 1;
  if constexpr (K <= 4) {
    // Few levels: the first wavefront sorts them in registers, lane p holding pattern p.  Its rank
    // is the number of levels below its own (ties by pattern); a lane-to-lane push then hands
    // every level to the lane of its rank, and thresholds, spread patterns and the pair table
    // follow without a barrier.
    if (tid < kWave) {
      const int pat = tid;
      float lv = 0.0f;
#pragma unroll
      for (int j = 0; j < K; ++j) lv = __fadd_rn(lv, ((pat >> j) & 1) ? alpha[j] : -alpha[j]);
      int rank = 0;
#pragma unroll
      for (int q = 0; q < P; ++q) {
        const float o = u32_as_f32(uint32_t(__builtin_amdgcn_readlane(int(f32_as_u32(lv)), q)));
        rank += (o < lv || (o == lv && q < pat)) ? 1 : 0;
      }
      if (pat >= P) rank = pat;  // idle lanes push to themselves
      const float lv_s = u32_as_f32(uint32_t(__builtin_amdgcn_ds_permute(rank * 4, int(f32_as_u32(lv)))));
      const uint32_t pat_s = uint32_t(__builtin_amdgcn_ds_permute(rank * 4, pat));
      const float lv_next = u32_as_f32(uint32_t(__builtin_amdgcn_ds_bpermute(((tid + 1) & (kWave - 1)) * 4,
                                                                            int(f32_as_u32(lv_s)))));
      const float tau = tid < P - 1 ? __fmul_rn(0.5f, __fadd_rn(lv_s, lv_next)) : __builtin_inff();
      uint32_t sp = 0;
#pragma unroll
      for (int bb = 0; bb < K; ++bb) sp |= ((pat_s >> bb) & 1u) << (8 * bb);
      if (tid < 3 * P) tb.tau[tid] = tau;  // 3P <= 48 lanes: thresholds, then +inf padding
      if (tid < P) {
        tb.lv_sorted[tid] = lv_s;
        tb.pat_sorted[tid] = pat_s;
        tb.spread[tid] = sp;
      }
      if (tid <= P + 1) {
        tb.pair[2 * tid] = f32_as_u32(tau);  // tau[P-1], tau[P], tau[P+1] are +inf
        tb.pair[2 * tid + 1] = tid < P ? sp : 0u;
      }
    }
    __syncthreads();
    // bucket table: the P-1 thresholds sit in registers, a bucket's lo is P-1 compares
    float t[P - 1];
#pragma unroll
    for (int i = 0; i < P - 1; ++i) t[i] = tb.tau[i];
    mymax = build_bucket_table<TB::LUT_SHIFT>(tb.lut, [&](float vmin) {
      int l = 0;
#pragma unroll
      for (int i = 0; i < P - 1; ++i) l += (t[i] < vmin) ? 1 : 0;
      return l;
    });
  } else {
    build_levels<K>(alpha, tb.lv_raw, tb.lv_sorted, tb.pat_sorted);
    for (int i = tid; i < 3 * P; i += nthr)
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
    // bucket table: tau[0..P-1) is sorted and tau[P-1] = +inf, so a branch-free binary search over
    // P entries finds lo
    mymax = build_bucket_table<TB::LUT_SHIFT>(tb.lut, [&](float vmin) {
      int l = 0;
#pragma unroll
      for (int s = P >> 1; s >= 1; s >>= 1) l += (tb.tau[l + s - 1] < vmin) ? s : 0;
      return l;
    });
  }
  if (mymax > 1) atomicMax(&tb.maxcnt, mymax);
  __syncthreads();
}

// Sum of NS per-thread float64 values over the threads of a workgroup, in a fixed order (so the
// result does not depend on timing): every wavefront adds its 64 lanes with register-to-register
// lane exchanges, lane 0 parks the NS wave totals in local memory, and thread s < NS adds the
// wavefronts' totals of statistic s in wavefront order.  On return thread s < NS holds total s
// (other threads: unspecified).  Ends with the buffer free for reuse after one more barrier.
struct WaveTotals {
  double v[kMaxWaves][48];  // nstat_of(8) = 45 statistics at most
};
template <int NS>
__device__ __forceinline__ double block_sum_stats(const double (&sv)[NS], WaveTotals& buf) {
  static_assert(NS <= 48, "statistics per record");
  const int tid = threadIdx.x;
  const int wave = tid / kWave, lane = tid & (kWave - 1);
  const int nwaves = (blockDim.x + kWave - 1) / kWave;
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const double t = wave_sum(sv[s]);
    if (lane == 0) buf.v[wave][s] = t;
  }
  __syncthreads();
  double mine = 0.0;
  if (tid < NS) {
    mine = buf.v[0][tid];
    for (int w = 1; w < nwaves; ++w) mine += buf.v[w][tid];
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
// sums (at most 8*VEC terms) folded into the thread's float64 sums.  A lane whose item lies
// beyond its row group (the ragged end of the last wave-item of a group) carries a copy of the
// group's last item: it stores the same bytes to the same place and counts nothing.
template <int K, int VEC>
__device__ __forceinline__ void finish_item(const uint32_t (&acc)[VEC][(K + 3) / 4], const float (&h32)[K], float sx32,
                                            uint8_t* __restrict__ dst, bool counts, EncodeStats<K>& st) {
  constexpr int NDW = (VEC * K + 3) / 4;
  constexpr int CW = (VEC + 3) / 4;
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
    store_dwords_stream<NDW>(reinterpret_cast<uint32_t*>(dst), out);
  } else {
#pragma unroll
    for (int p = 0; p < K; ++p) dst[p] = uint8_t(acc[0][p / 4] >> (8 * (p % 4)));
  }
  // (selects, not a branch around the sums: with a branch the compiler moves the whole chain of
  // per-element adds of the item behind it, to the end of the round, and every row of x then
  // has to stay in registers until there)
  const uint32_t keep = counts ? 0xFFFFFFFFu : 0u;
  uint32_t pw[K][CW];  // plane bytes of all VEC columns, plane-major
#pragma unroll
  for (int p = 0; p < K; ++p) {
#pragma unroll
    for (int w = 0; w < CW; ++w) pw[p][w] = 0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) pw[p][c / 4] |= ((acc[c][p / 4] >> (8 * (p % 4))) & 0xFFu) << (8 * (c % 4));
#pragma unroll
    for (int w = 0; w < CW; ++w) pw[p][w] &= keep;
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
  st.Sx += double(counts ? sx32 : 0.0f);
#pragma unroll
  for (int p = 0; p < K; ++p) st.H[p] += double(counts ? h32[p] : 0.0f);
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
  finish_item<K, 1>(acc, h32, sx32, payload + ((g * m + j) * K), true, st);
}

// ---- the pipelined stream over complete row groups -------------------------------------------
// Unit of work = wave-item: 64 adjacent items (one per lane) of one row group, i.e. 8 rows x
// 64*VEC columns, every row a contiguous run in memory.  Wavefronts draw wave-items one at a
// time: a wavefront that is served faster (the instruction arbiter favours the oldest wavefront
// of a SIMD, some dies sit closer to the memory they happen to read) simply takes more of them,
// and the whole grid finishes together instead of waiting for its slowest compute unit.  The
// counters live in device memory, one per group of eight workgroups (one counter for the whole
// grid would see a request every nanosecond; an atomic on one address takes about twelve).
// Which wavefront ran which wave-item decides only the grouping of the float64 partial sums,
// never a payload bit.
//
// Queue position c of group i is wave-item (c / 64) * sweep + 64 * i + c % 64, sweep = 64 *
// groups: at any time the grid reads one contiguous stretch of each of eight rows (the pattern
// memory likes best), the groups advancing through the tensor side by side.
struct WorkQueue {
  uint32_t* counter;  // the group's counter: zero when the kernel starts, put back by the finalize kernel
  uint32_t first;     // 64 * group
  uint32_t sweep;     // wave-items all groups take per sweep
  uint32_t count;     // queue positions 0 .. count-1 exist
  uint32_t drawn;     // positions handed out without the counter: two per wavefront of the group
};
__device__ __forceinline__ uint32_t queue_to_wave_item(uint32_t c, const WorkQueue& q) {
  return (c / uint32_t(kGroupSlots)) * q.sweep + q.first + (c % uint32_t(kGroupSlots));
}

// Where a lane's item of a wave-item lives: the row group (the same in all lanes and kept in
// scalar registers, so that a row load is "scalar base + 32-bit lane offset" and costs no vector
// registers for its address) and the lane's own item number inside the group.
struct ItemAddr {
  uint32_t g;    // row group (scalar)
  uint32_t jv;   // item inside the group, clamped to the last one
  bool counts;   // false for the clamped copies that fill the ragged end of a row group
};
// Item of lane `lane` in wave-item w; wpg wave-items and ipg items per row group (both below
// 2^32, checked on the host, as are the byte lengths of a row of x and of a row group's planes).
__device__ __forceinline__ ItemAddr item_addr(uint32_t w, uint32_t wpg, uint32_t ipg, int lane) {
  ItemAddr a;
  a.g = uint32_t(__builtin_amdgcn_readfirstlane(int(w / wpg)));
  a.jv = (w - a.g * wpg) * uint32_t(kWave) + uint32_t(lane);
  a.counts = a.jv < ipg;
  if (!a.counts) a.jv = ipg - 1u;
  return a;
}
// Row 8g + r of the item: the base is formed from scalars only; lane_x = jv * VEC * sizeof(T).
template <typename T, int VEC>
__device__ __forceinline__ RawRow<VEC> load_row(const T* __restrict__ x, uint32_t g, uint64_t row_bytes, int r,
                                                uint32_t lane_x) {
  const char* base = reinterpret_cast<const char*>(x) + (uint64_t(g) * 8u + uint64_t(r)) * row_bytes;
  return load_raw<T, VEC>(reinterpret_cast<const T*>(base + lane_x));
}

template <typename T, int K, int VEC, int MC>
__device__ __forceinline__ void encode_stream(const EncodeTables<K>& tb, const T* __restrict__ x,
                                              uint8_t* __restrict__ payload, uint64_t m, uint32_t ipg, uint32_t wpg,
                                              const WorkQueue& q, uint32_t cur, uint32_t nxt, ItemAddr ca,
                                              RawRow<VEC> (&fr)[8], EncodeStats<K>& st) {
  constexpr int NW = (K + 3) / 4;
  constexpr int GR = VEC >= 4 ? 1 : 4 / VEC;  // rows whose table lookups are issued together (at least 4 elements)
  const int lane = threadIdx.x & (kWave - 1);
  const uint64_t row_bytes = m * sizeof(T);
  // The first item's rows have had the whole table build to arrive.  Waiting for them here
  // (vmcnt 0, the other counters untouched) gives the loop an empty set of outstanding loads
  // on entry whatever code precedes it, so that the waits the compiler places inside the loop
  // are the ones its own steady state needs and no more.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  while (cur < q.count) {
    // the wave-item after the next: asked for now, looked at when this item is done (the answer
    // comes back in line with the row loads issued below, well before it is needed)
    uint32_t after_v = 0;
    if (lane == 0) after_v = __hip_atomic_fetch_add(q.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // When there is no next wave-item every lane re-reads the first item of the tensor (valid,
    // one cache line per row for the whole wavefront), so that the loads stay unconditional and
    // the compiler can reuse the row registers in place.
    ItemAddr na;
    na.g = 0; na.jv = 0; na.counts = false;
    if (nxt < q.count) na = item_addr(queue_to_wave_item(nxt, q), wpg, ipg, lane);
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
      // The loads of the next item's rows go where this group's rows were: they may not be
      // issued before the last use of those registers (else the compiler keeps a second set of
      // row registers and copies it over at the end of the round, which also means waiting for
      // all eight loads there).
      __builtin_amdgcn_sched_barrier(0);
      {
        // the lane offset passes through an empty asm, so that the addresses of this group's loads
        // are formed here and not, all eight of them, at the top of the round
        uint32_t lane_x = na.jv * uint32_t(VEC * sizeof(T));
        asm volatile("" : "+v"(lane_x));
#pragma unroll
        for (int rr = 0; rr < GR; ++rr) fr[r0 + rr] = load_row<T, VEC>(x, na.g, row_bytes, r0 + rr, lane_x);
      }
      // keep the instruction scheduler from mixing groups: it would otherwise hoist the table
      // reads of all 8*VEC elements and run out of registers
      __builtin_amdgcn_sched_barrier(0);
    }
    finish_item<K, VEC>(acc, h32, sx32, payload + uint64_t(ca.g) * m * uint32_t(K) + ca.jv * uint32_t(VEC * K), ca.counts,
                        st);
    cur = nxt;
    nxt = q.drawn + uint32_t(__builtin_amdgcn_readfirstlane(int(after_v)));
    ca = na;
  }
}

// ========================================================================= finalize (M5)
// From the call's totals: alpha_cur = (B^T B)^-1 B^T x by Gaussian elimination with row
// pivoting, the moving average with beta = min(0.9, (1+t)/(10+t)), m_q = mean(B alpha_t - x);
// header = [alpha_t, m_q].  One thread; K is a template parameter so that the k x k system
// lives in registers.  tot: sums of x over the +1 entries of each plane, sum of x, +1 counts
// per plane, disagreement counts per plane pair.
template <int K>
__device__ __forceinline__ void solve_and_write_header(const double* tot, const float (&alpha_prev)[K], double n_elems,
                                                       double beta, float* __restrict__ header) {
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
  double dot = 0.0;
#pragma unroll
  for (int p = 0; p < K; ++p) {
    const float a_t = float(beta * a_prev[p] + (1.0 - beta) * (singular ? a_prev[p] : cur[p]));
    header[p] = a_t;
    dot += double(a_t) * Sb[p];
  }
  header[K] = float((dot - Sx) / n_elems);
}

// What the kernels of one compress call share: the per-workgroup records in the workspace
// (stat-major: statistic s of workgroup b at records[s * nrec + b]), the previous coefficients
// and the header to write.
struct MbqCall {
  uint32_t* counters;  // work counters of the encode kernel (control block of the workspace)
  double* records;
  const float* alpha_prev;
  float* header;
  double n_elems;
  double beta;  // weight of the previous coefficients in the moving average: min(0.9, (1+t)/(10+t))
};

// End of an encode kernel (M4): the workgroup adds up its threads' statistics in a fixed order
// and stores one record.
template <int K>
__device__ __forceinline__ void store_record(const EncodeStats<K>& st, const MbqCall& call, WaveTotals& buf) {
  constexpr int NPAIR = K * (K - 1) / 2;
  constexpr int NSTAT = nstat_of(K);
  double sv[NSTAT];
#pragma unroll
  for (int p = 0; p < K; ++p) sv[p] = st.H[p];
  sv[K] = st.Sx;
#pragma unroll
  for (int p = 0; p < K; ++p) sv[K + 1 + p] = double(st.cnt[p]);
#pragma unroll
  for (int i = 0; i < NPAIR; ++i) sv[2 * K + 1 + i] = double(st.dis[i]);
  const double total = block_sum_stats<NSTAT>(sv, buf);
  if (threadIdx.x < NSTAT) call.records[int64_t(threadIdx.x) * gridDim.x + blockIdx.x] = total;
}

// M5, one workgroup: thread b takes records b, b + 256, ... of every statistic (all loads of a
// round issued before their adds), the workgroup adds them up in the same fixed order, one
// thread solves and writes the header.
template <int K>
__global__ __launch_bounds__(kBlock) void mbq_finalize_kernel(MbqCall call, int nrec) {
  constexpr int NSTAT = nstat_of(K);
  __shared__ WaveTotals red;
  __shared__ double tot[48];
  const int tid = threadIdx.x;
  float alpha_prev[K];  // asked for together with the records: the solve at the end would otherwise wait for them
#pragma unroll
  for (int p = 0; p < K; ++p) alpha_prev[p] = call.alpha_prev[p];
  double a[NSTAT];
#pragma unroll
  for (int s = 0; s < NSTAT; ++s) a[s] = 0.0;
  for (int b = tid; b < nrec; b += kBlock) {
    double v[NSTAT];
#pragma unroll
    for (int s = 0; s < NSTAT; ++s) v[s] = call.records[int64_t(s) * nrec + b];
#pragma unroll
    for (int s = 0; s < NSTAT; ++s) a[s] += v[s];
  }
  const double total = block_sum_stats<NSTAT>(a, red);
  if (tid < NSTAT) tot[tid] = total;
  if (tid < kMaxGroups) call.counters[tid * kCounterStride] = 0u;  // the encode kernel's work counters, for the next call
  __syncthreads();
  if (tid == 0) solve_and_write_header<K>(tot, alpha_prev, call.n_elems, call.beta, call.header);
}

// Fused M1..M4.  Complete row groups go through the pipelined stream: row r of the next
// wave-item is requested as soon as row r of the current one has been consumed, so a wavefront
// always has loads in flight while it works; the first wave-item's rows are requested before
// the tables are built.  The last, partial row group (n % 8 != 0) and the rare case of more
// than two thresholds per bucket take the plain path, one column per thread.
template <typename T, int K, int VEC>
__global__ __launch_bounds__(kEncBlock) void mbq_encode_kernel(const T* __restrict__ x, uint8_t* __restrict__ payload,
                                                               MbqCall call, int64_t n, int64_t m, uint32_t ipg,
                                                               uint32_t wpg, uint32_t n_wave_items) {
  constexpr int NPAIR = K * (K - 1) / 2;
  __shared__ EncodeTables<K> tb;
  __shared__ WaveTotals red;

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  float alpha[K];  // asked for first: nothing below needs them before the tables are built
#pragma unroll
  for (int j = 0; j < K; ++j) alpha[j] = call.alpha_prev[j];
  // this wavefront's place in its group's queue: the first two positions of every wavefront are
  // fixed (its index among the group's wavefronts, and that plus their number), the rest are drawn
  WorkQueue q;
  const uint32_t group = blockIdx.x / uint32_t(kGroupBlocks);
  const uint32_t groups = (gridDim.x + uint32_t(kGroupBlocks) - 1u) / uint32_t(kGroupBlocks);
  const uint32_t group_blocks =
      gridDim.x - group * uint32_t(kGroupBlocks) < uint32_t(kGroupBlocks) ? gridDim.x - group * uint32_t(kGroupBlocks)
                                                                        : uint32_t(kGroupBlocks);
  const uint32_t group_waves = group_blocks * uint32_t(kEncWaves);
  q.counter = call.counters + group * uint32_t(kCounterStride);
  q.first = group * uint32_t(kGroupSlots);
  q.sweep = groups * uint32_t(kGroupSlots);
  {
    const uint32_t full_sweeps = n_wave_items / q.sweep;
    const uint32_t rest = n_wave_items - full_sweeps * q.sweep;
    const uint32_t extra =
        rest > q.first ? (rest - q.first < uint32_t(kGroupSlots) ? rest - q.first : uint32_t(kGroupSlots)) : 0u;
    q.count = full_sweeps * uint32_t(kGroupSlots) + extra;
  }
  q.drawn = 2u * group_waves;
  const uint32_t cur = uint32_t(__builtin_amdgcn_readfirstlane(
      int((blockIdx.x - group * uint32_t(kGroupBlocks)) * uint32_t(kEncWaves) + uint32_t(tid) / uint32_t(kWave))));
  const uint32_t nxt = cur + group_waves;
  RawRow<VEC> fr[8];
  ItemAddr ca;
  ca.g = 0; ca.jv = 0; ca.counts = false;
  if (cur < q.count) {
    ca = item_addr(queue_to_wave_item(cur, q), wpg, ipg, lane);
#pragma unroll
    for (int r = 0; r < 8; ++r)
      fr[r] = load_row<T, VEC>(x, ca.g, uint64_t(m) * sizeof(T), r, ca.jv * uint32_t(VEC * sizeof(T)));
  }

  build_encode_tables<K>(alpha, tb);
  // the same value in every lane: read it into a scalar register, so that the choice of path
  // below is a scalar branch and not a divergent one whose sides run one after the other
  const int maxcnt = __builtin_amdgcn_readfirstlane(tb.maxcnt);

  EncodeStats<K> st;
  st.Sx = 0.0;
#pragma unroll
  for (int p = 0; p < K; ++p) { st.H[p] = 0.0; st.cnt[p] = 0; }
#pragma unroll
  for (int i = 0; i < (NPAIR > 0 ? NPAIR : 1); ++i) st.dis[i] = 0;

  const int64_t stride = int64_t(gridDim.x) * kEncBlock;
  const int64_t gtid = int64_t(blockIdx.x) * kEncBlock + tid;
  const bool stream = n_wave_items != 0u;  // else: a geometry too narrow for wave-items
  if (stream && maxcnt == 1) {
    encode_stream<T, K, VEC, 1>(tb, x, payload, uint64_t(m), ipg, wpg, q, cur, nxt, ca, fr, st);
  } else if (stream && maxcnt == 2 && K <= 4) {
    encode_stream<T, K, VEC, 2>(tb, x, payload, uint64_t(m), ipg, wpg, q, cur, nxt, ca, fr, st);
  } else {
    // several thresholds share a bucket (levels closer than a bucket's width), or a very narrow
    // tensor: rare.  One column per thread keeps this path's register needs out of the kernel's
    // budget.
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
  store_record<K>(st, call, red);
}

// ================================================ comparison layout: one byte per binary base
// ACCEPT_LAYOUT_UNENCODED: B itself, +1 / -1 as bytes, element-major with the k bases
// innermost ("w/o enc." in the paper's size table).  Same levels, same sums and the same
// finalize kernel as the bit-plane path; plain flat loops, four elements per thread and step.
template <typename T, int K>
__global__ __launch_bounds__(kBlock) void mbq_encode_plain_kernel(const T* __restrict__ x,
                                                                  uint8_t* __restrict__ payload, MbqCall call,
                                                                  int64_t N) {
  constexpr int NW = (K + 3) / 4;
  constexpr int NPAIR = K * (K - 1) / 2;
  __shared__ EncodeTables<K> tb;
  __shared__ WaveTotals red;
  const float* alpha_prev = call.alpha_prev;
  const int tid = threadIdx.x;
  float alpha[K];
#pragma unroll
  for (int j = 0; j < K; ++j) alpha[j] = alpha_prev[j];
  build_encode_tables<K>(alpha, tb);
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
  store_record<K>(st, call, red);
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

// ======================================================= residue initialisation (batch 0)
// rho_0 = x, b_j = sign(rho_j) (sign(0) = +1), alpha_j = mean|rho_j|, rho_(j+1) = rho_j - alpha_j b_j,
// carried in float64 like the definition.  alpha_j needs the whole tensor's |rho_j|, so the method
// is k passes over x; pass j reads alpha_0..alpha_(j-1) from device memory.

// rho_j of one element.
__device__ __forceinline__ double residue(float x, const double (&a)[8], int j) {
  double rho = double(x);
  for (int q = 0; q < j; ++q) rho -= (rho >= 0.0) ? a[q] : -a[q];
  return rho;
}

// Pass j, sums only: sum of |rho_j|, 16-byte streaming loads, four in flight per thread; one
// record (a single float64) per workgroup.
template <typename T>
__global__ __launch_bounds__(kBlock) void mbq_init_pass_kernel(const T* __restrict__ x, int64_t N, int j,
                                                                const float* __restrict__ alpha,
                                                                double* __restrict__ records) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int UNROLL = 4;
  __shared__ WaveTotals red;
  double a[8];
  for (int i = 0; i < 8; ++i) a[i] = i < j ? double(alpha[i]) : 0.0;
  const int64_t nvec = N / VEC;
  const int64_t stride = int64_t(gridDim.x) * kBlock;
  double acc = 0.0;
  int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  for (; v + (UNROLL - 1) * stride < nvec; v += UNROLL * stride) {
    float f[UNROLL][VEC];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) load_vec_stream(x + (v + u * stride) * VEC, f[u]);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc += fabs(residue(f[u][e], a, j));
  }
  for (; v < nvec; v += stride) {
    float f[VEC];
    load_vec_stream(x + v * VEC, f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc += fabs(residue(f[e], a, j));
  }
  if (blockIdx.x == 0 && int64_t(threadIdx.x) < N - nvec * VEC)
    acc += fabs(residue(load_one(x + nvec * VEC + threadIdx.x), a, j));
  const double sv[1] = {acc};
  const double total = block_sum_stats<1>(sv, red);
  if (threadIdx.x == 0) records[blockIdx.x] = total;
}

// Last pass (j = K-1) of a batch-0 compression: the signs b_0..b_(K-1) of every element need
// only alpha_0..alpha_(K-2), so the bit planes of B^0 are written in the same pass that adds up
// |rho_(K-1)| for alpha_(K-1).  Items as in the encoder (8 rows x VEC columns per lane, row loads
// contiguous across lanes), static grid-stride assignment.  Record per workgroup: sum|rho_(K-1)|,
// sum of x, +1 counts of the K planes.
template <typename T, int K, int VEC>
__global__ __launch_bounds__(kBlock) void mbq_init_encode_kernel(const T* __restrict__ x,
                                                                  const float* __restrict__ alpha,
                                                                  uint8_t* __restrict__ payload,
                                                                  double* __restrict__ records, int64_t n, int64_t m,
                                                                  int64_t ipg, int64_t items, ItemStep step) {
  constexpr int NW = (K + 3) / 4;
  constexpr int NDW = (VEC * K + 3) / 4;
  constexpr int NS = K + 2;
  __shared__ WaveTotals red;
  double a[8];
  for (int i = 0; i < 8; ++i) a[i] = i < K - 1 ? double(alpha[i]) : 0.0;
  double sum_abs = 0.0, sum_x = 0.0;
  uint32_t cnt[K];
#pragma unroll
  for (int p = 0; p < K; ++p) cnt[p] = 0;
  int64_t it = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  ItemPos pos;
  pos.g = it / ipg;
  pos.jv = it - pos.g * ipg;
  for (; it < items; it += int64_t(gridDim.x) * kBlock, item_advance(pos, step, ipg)) {
    const int64_t row0 = pos.g * 8;
    const int nrows = (n - row0) < 8 ? int(n - row0) : 8;
    const T* xc = x + row0 * m + pos.jv * VEC;
    RawRow<VEC> fr[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {  // all row loads first, so that they overlap
      if constexpr (VEC > 1) fr[r].v = make_uint4(0u, 0u, 0u, 0u); else fr[r].v = 0u;
      if (r < nrows) fr[r] = load_raw<T, VEC>(xc + r * m);
    }
    uint32_t acc[VEC][NW];
#pragma unroll
    for (int c = 0; c < VEC; ++c)
#pragma unroll
      for (int w = 0; w < NW; ++w) acc[c][w] = 0;
    float sx32 = 0.0f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      float row[VEC];
      widen_raw<VEC>(fr[r], row);
#pragma unroll
      for (int c = 0; c < VEC; ++c) {
        // the recurrence of residue(), keeping every sign on the way
        double rho = double(row[c]);
        uint32_t sp[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) sp[w] = 0;
#pragma unroll
        for (int q = 0; q < K; ++q) {
          const bool pos_sign = rho >= 0.0;
          sp[q / 4] |= (pos_sign ? 1u : 0u) << (8 * (q % 4));
          if (q < K - 1) rho -= pos_sign ? a[q] : -a[q];
        }
        const bool have = r < nrows;  // a missing row contributes 0 bits and nothing to the sums
        sum_abs += have ? fabs(rho) : 0.0;
        sx32 = __fadd_rn(sx32, have ? row[c] : 0.0f);
#pragma unroll
        for (int w = 0; w < NW; ++w) acc[c][w] = (acc[c][w] << 1) | (have ? sp[w] : 0u);
      }
    }
    sum_x += double(sx32);
#pragma unroll
    for (int p = 0; p < K; ++p)
#pragma unroll
      for (int c = 0; c < VEC; ++c) cnt[p] += __popc((acc[c][p / 4] >> (8 * (p % 4))) & 0xFFu);
    uint8_t* dst = payload + ((pos.g * m + pos.jv * VEC) * K);
    if constexpr (VEC > 1) {
      uint32_t out[NDW];
#pragma unroll
      for (int w = 0; w < NDW; ++w) out[w] = 0;
#pragma unroll
      for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int p = 0; p < K; ++p) {
          const int b = c * K + p;
          out[b / 4] |= ((acc[c][p / 4] >> (8 * (p % 4))) & 0xFFu) << (8 * (b % 4));
        }
      store_dwords<NDW>(reinterpret_cast<uint32_t*>(dst), out);
    } else {
#pragma unroll
      for (int p = 0; p < K; ++p) dst[p] = uint8_t(acc[0][p / 4] >> (8 * (p % 4)));
    }
  }
  double sv[NS];
  sv[0] = sum_abs;
  sv[1] = sum_x;
#pragma unroll
  for (int p = 0; p < K; ++p) sv[2 + p] = double(cnt[p]);
  const double total = block_sum_stats<NS>(sv, red);
  if (threadIdx.x < NS) records[int64_t(threadIdx.x) * gridDim.x + blockIdx.x] = total;
}

// After pass j: alpha_j = (sum of the workgroups' |rho_j| sums) / N, written to alpha_out[j].
// After the last pass of a batch-0 compression (nstat = k + 2) also the rest of the header:
// m_q = mean(B^0 alpha^0 - x) = (sum_p alpha_p (2 cnt_p - N) - sum x) / N  (eq. (biased error)),
// written behind the k coefficients that the earlier passes left in alpha_out.
__global__ __launch_bounds__(kBlock) void mbq_init_finalize_kernel(const double* __restrict__ records, int nrec,
                                                                    int nstat, double n_elems, int j,
                                                                    float* __restrict__ alpha_out) {
  __shared__ WaveTotals red;
  __shared__ double tot[16];
  const int tid = threadIdx.x;
  for (int s = 0; s < nstat; ++s) {
    double a = 0.0;
    for (int b = tid; b < nrec; b += kBlock) a += records[int64_t(s) * nrec + b];
    const double sv[1] = {a};
    const double total = block_sum_stats<1>(sv, red);
    if (tid == 0) tot[s] = total;
    __syncthreads();  // the buffer of the workgroup sum is free again
  }
  if (tid != 0) return;
  const float a_j = float(tot[0] / n_elems);
  alpha_out[j] = a_j;
  if (nstat > 1) {
    const int k = nstat - 2;
    double dot = 0.0;
    for (int p = 0; p < k; ++p) {
      const double a_p = p == j ? double(a_j) : double(alpha_out[p]);
      dot += a_p * (2.0 * tot[2 + p] - n_elems);
    }
    alpha_out[k] = float((dot - tot[1]) / n_elems);
  }
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

MbqCall make_call(const accept_desc& d, const float* alpha_prev, void* header, void* ws) {
  MbqCall c;
  c.counters = static_cast<uint32_t*>(ws);
  c.records = reinterpret_cast<double*>(static_cast<char*>(ws) + kCtrlBytes);
  c.alpha_prev = alpha_prev;
  c.header = static_cast<float*>(header);
  c.n_elems = double(d.n) * double(d.m);
  const double beta = (1.0 + double(d.t)) / (10.0 + double(d.t));  // eq. (alpha update)
  c.beta = beta > 0.9 ? 0.9 : beta;
  return c;
}

template <typename T, int K, int VEC>
hipError_t launch_encode(const accept_desc& d, const MPlan& p, const T* x, uint8_t* payload, const MbqCall& call,
                         hipStream_t s) {
  hipLaunchKernelGGL((mbq_encode_kernel<T, K, VEC>), dim3(p.grid), dim3(kEncBlock), 0, s, x, payload, call, d.n, d.m,
                     uint32_t(p.stream ? d.m / VEC : 1), p.wpg, p.n_wave_items);
  return hipGetLastError();
}

template <typename T, int VEC>
hipError_t encode_k(const accept_desc& d, const MPlan& p, const T* x, uint8_t* payload, const MbqCall& call,
                    hipStream_t s) {
  switch (d.bits) {
    case 1: return launch_encode<T, 1, VEC>(d, p, x, payload, call, s);
    case 2: return launch_encode<T, 2, VEC>(d, p, x, payload, call, s);
    case 3: return launch_encode<T, 3, VEC>(d, p, x, payload, call, s);
    case 4: return launch_encode<T, 4, VEC>(d, p, x, payload, call, s);
    case 5: return launch_encode<T, 5, VEC>(d, p, x, payload, call, s);
    case 6: return launch_encode<T, 6, VEC>(d, p, x, payload, call, s);
    case 7: return launch_encode<T, 7, VEC>(d, p, x, payload, call, s);
    case 8: return launch_encode<T, 8, VEC>(d, p, x, payload, call, s);
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

template <typename T, int K, int VEC>
hipError_t launch_init_encode(const accept_desc& d, const T* x, const float* alpha, uint8_t* payload, double* records,
                              int grid, hipStream_t s) {
  const int64_t ipg = d.m / VEC;
  const int64_t items = ((d.n + 7) / 8) * ipg;
  hipLaunchKernelGGL((mbq_init_encode_kernel<T, K, VEC>), dim3(grid), dim3(kBlock), 0, s, x, alpha, payload, records,
                     d.n, d.m, ipg, items, step_for(grid, ipg));
  return hipGetLastError();
}

template <typename T, int VEC>
hipError_t init_encode_k(const accept_desc& d, const T* x, const float* alpha, uint8_t* payload, double* records,
                         int grid, hipStream_t s) {
  switch (d.bits) {
    case 1: return launch_init_encode<T, 1, VEC>(d, x, alpha, payload, records, grid, s);
    case 2: return launch_init_encode<T, 2, VEC>(d, x, alpha, payload, records, grid, s);
    case 3: return launch_init_encode<T, 3, VEC>(d, x, alpha, payload, records, grid, s);
    case 4: return launch_init_encode<T, 4, VEC>(d, x, alpha, payload, records, grid, s);
    case 5: return launch_init_encode<T, 5, VEC>(d, x, alpha, payload, records, grid, s);
    case 6: return launch_init_encode<T, 6, VEC>(d, x, alpha, payload, records, grid, s);
    case 7: return launch_init_encode<T, 7, VEC>(d, x, alpha, payload, records, grid, s);
    case 8: return launch_init_encode<T, 8, VEC>(d, x, alpha, payload, records, grid, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

MPlan make_mplan(const accept_desc& d) {
  MPlan p{};
  p.vec = vec_for(d.in_dtype, d.m);
  p.G = (d.n + 7) / 8;
  p.items = p.G * (d.m / p.vec);
  // The pipelined stream of the encode kernel works on wave-items (64 items of one row group).
  // It needs at least one full wave-item per row group to be worth it and 32-bit wave-item
  // numbers; other geometries (very narrow tensors) go one column per thread.
  const int64_t ipg = d.m / p.vec;
  const int64_t wpg = (ipg + kWave - 1) / kWave;
  const int64_t full_groups = d.n / 8;
  const int64_t wave_items = full_groups * wpg;
  p.stream = full_groups > 0 && ipg >= kWave && wave_items < (int64_t(1) << 31) && d.m * 8 < (int64_t(1) << 32);
  p.wpg = p.stream ? uint32_t(wpg) : 1u;
  p.n_wave_items = p.stream ? uint32_t(wave_items) : 0u;
  {
    // one workgroup of 8 wavefronts per compute unit at most; fewer when there is less work
    int64_t blocks = p.stream ? (wave_items + kEncWaves - 1) / kEncWaves
                              : (full_groups * d.m + kEncBlock - 1) / kEncBlock;
    const int64_t tail_blocks = (d.n % 8 != 0) ? (d.m + kEncBlock - 1) / kEncBlock : 0;
    if (blocks < tail_blocks) blocks = tail_blocks;
    if (blocks < 1) blocks = 1;
    p.grid = int(blocks < kEncodeGridMax ? blocks : kEncodeGridMax);
  }
  p.nstat = nstat_of(d.bits);
  // control block, then room for kMaxRecords records of the widest kind (k = 8)
  const size_t bytes = kCtrlBytes + size_t(nstat_of(8)) * kMaxRecords * sizeof(double);
  p.bytes = (bytes + 255) / 256 * 256;
  return p;
}

template <typename T>
hipError_t encode_plain_k(const accept_desc& d, int grid, const T* x, uint8_t* payload, const MbqCall& call,
                          hipStream_t s) {
  const int64_t N = d.n * d.m;
#define ACCEPT_ENC(KK)                                                                                         \
  case KK:                                                                                                     \
    hipLaunchKernelGGL((mbq_encode_plain_kernel<T, KK>), dim3(grid), dim3(kBlock), 0, s, x, payload, call, N); \
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
  const MbqCall call = make_call(d, alpha_prev, header, ws);
  uint8_t* pl = static_cast<uint8_t*>(payload);
  hipError_t e;
  mark(tm, s);
  int nrec = p.grid;
  if (d.layout == ACCEPT_LAYOUT_UNENCODED) {
    const int grid = nrec = grid_for(d.n * d.m / 4 + 4, kPlainGridMax);
    e = d.in_dtype == ACCEPT_BF16 ? encode_plain_k<bf16_t>(d, grid, static_cast<const bf16_t*>(x), pl, call, s)
                                  : encode_plain_k<float>(d, grid, static_cast<const float*>(x), pl, call, s);
  } else if (d.in_dtype == ACCEPT_BF16) {
    const bf16_t* xb = static_cast<const bf16_t*>(x);
    e = p.vec == 8 ? encode_k<bf16_t, 8>(d, p, xb, pl, call, s) : encode_k<bf16_t, 1>(d, p, xb, pl, call, s);
  } else {
    const float* xf = static_cast<const float*>(x);
    e = p.vec == 4 ? encode_k<float, 4>(d, p, xf, pl, call, s) : encode_k<float, 1>(d, p, xf, pl, call, s);
  }
  if (e != hipSuccess) return e;
  mark(tm, s);
#define ACCEPT_FIN(KK)                                                                          \
  case KK:                                                                                      \
    hipLaunchKernelGGL(mbq_finalize_kernel<KK>, dim3(1), dim3(kBlock), 0, s, call, nrec);       \
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

// Residue initialisation.  payload == nullptr: k sum passes, alpha^0 to alpha_out[0..k).
// Otherwise a batch-0 compression: k - 1 sum passes and one pass that also writes the bit planes
// of B^0 to payload; alpha_out is then the header, [alpha^0, m_q].
hipError_t launch_mbq_init(const accept_desc& d, const MPlan& p, const void* x, float* alpha_out, void* payload,
                           void* ws, hipStream_t s) {
  double* records = reinterpret_cast<double*>(static_cast<char*>(ws) + kCtrlBytes);
  const int64_t N = d.n * d.m;
  const int k = d.bits;
  const bool bf = d.in_dtype == ACCEPT_BF16;
  const int grid = grid_for(N / (bf ? 8 : 4) / 4 + 1, kInitGrid);
  hipError_t e;
  for (int j = 0; j < k; ++j) {
    const bool planes = payload != nullptr && j == k - 1;
    int nrec = grid, nstat = 1;
    if (planes) {
      nrec = grid_for(p.items, kPlainGridMax);
      nstat = k + 2;
      uint8_t* pl = static_cast<uint8_t*>(payload);
      if (bf) {
        const bf16_t* xb = static_cast<const bf16_t*>(x);
        e = p.vec == 8 ? init_encode_k<bf16_t, 8>(d, xb, alpha_out, pl, records, nrec, s)
                       : init_encode_k<bf16_t, 1>(d, xb, alpha_out, pl, records, nrec, s);
      } else {
        const float* xf = static_cast<const float*>(x);
        e = p.vec == 4 ? init_encode_k<float, 4>(d, xf, alpha_out, pl, records, nrec, s)
                       : init_encode_k<float, 1>(d, xf, alpha_out, pl, records, nrec, s);
      }
    } else {
      if (bf)
        hipLaunchKernelGGL((mbq_init_pass_kernel<bf16_t>), dim3(grid), dim3(kBlock), 0, s,
                           static_cast<const bf16_t*>(x), N, j, alpha_out, records);
      else
        hipLaunchKernelGGL((mbq_init_pass_kernel<float>), dim3(grid), dim3(kBlock), 0, s, static_cast<const float*>(x),
                           N, j, alpha_out, records);
      e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mbq_init_finalize_kernel, dim3(1), dim3(kBlock), 0, s, records, nrec, nstat, double(N), j,
                       alpha_out);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace accept
