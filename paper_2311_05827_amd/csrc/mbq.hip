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
// finished plane bytes, B^T x from masked adds.
#include "common.hpp"

namespace accept {

namespace {

constexpr int kEncodeGridMax = 2048;
constexpr int kDecodeGridMax = 8192;
constexpr int kInitGrid = 1024;

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
template <typename T, int K, int VEC>
__global__ __launch_bounds__(kBlock) void mbq_encode_kernel(const T* __restrict__ x,
                                                             const float* __restrict__ alpha_prev,
                                                             uint8_t* __restrict__ payload,
                                                             double* __restrict__ partials, int64_t n, int64_t m,
                                                             int64_t ipg, int64_t items, ItemStep step) {
  constexpr int P = 1 << K;
  constexpr int NW = (K + 3) / 4;            // 32-bit words of a spread pattern
  constexpr int NPAIR = K * (K - 1) / 2;
  constexpr int NSTAT = nstat_of(K);
  constexpr int NDW = (VEC * K + 3) / 4;     // output dwords per item (VEC >= 4)
  __shared__ float lv_raw[P];
  __shared__ float lv_sorted[P];
  __shared__ uint32_t pat_sorted[P];
  __shared__ float tau[P];
  __shared__ uint32_t spread[NW][P];
  __shared__ double red[kBlock / kWave][NSTAT];

  const int tid = threadIdx.x;
  build_levels<K>(alpha_prev, lv_raw, lv_sorted, pat_sorted);
  if (tid < P) {
    // thresholds: float32 midpoints of neighbouring levels; entry P-1 is never read
    tau[tid] = (tid < P - 1) ? __fmul_rn(0.5f, __fadd_rn(lv_sorted[tid], lv_sorted[tid + 1])) : 0.0f;
    const uint32_t pat = pat_sorted[tid];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      uint32_t sp = 0;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if (4 * w + b < K) sp |= ((pat >> (4 * w + b)) & 1u) << (8 * b);
      spread[w][tid] = sp;
    }
  }
  __syncthreads();

  double A[K];       // sum of x over elements whose plane-p sign is +1
  double Sx = 0.0;   // sum of x
  uint32_t cnt[K];   // number of +1 signs per plane
  uint32_t dis[NPAIR > 0 ? NPAIR : 1];  // number of elements whose planes p<q disagree
#pragma unroll
  for (int p = 0; p < K; ++p) { A[p] = 0.0; cnt[p] = 0; }
#pragma unroll
  for (int i = 0; i < (NPAIR > 0 ? NPAIR : 1); ++i) dis[i] = 0;

  int64_t it = int64_t(blockIdx.x) * kBlock + tid;
  ItemPos pos;
  pos.g = it / ipg;
  pos.jv = it - pos.g * ipg;
  for (; it < items; it += int64_t(gridDim.x) * kBlock, item_advance(pos, step, ipg)) {
    const int64_t row0 = pos.g * 8;
    const T* xc = x + pos.jv * VEC;
    float f[8][VEC];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      if (row0 + r < n) {
        if constexpr (VEC > 1) {
          load_vec(xc + (row0 + r) * m, f[r]);
        } else {
          f[r][0] = load_one(xc + (row0 + r) * m);
        }
      } else {
#pragma unroll
        for (int c = 0; c < VEC; ++c) f[r][c] = 0.0f;
      }
    }
    uint32_t acc[VEC][NW];
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
#pragma unroll
      for (int w = 0; w < NW; ++w) acc[c][w] = 0;
      float a32[K];
      float sx32 = 0.0f;
#pragma unroll
      for (int p = 0; p < K; ++p) a32[p] = 0.0f;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        uint32_t sp[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) sp[w] = 0;
        if (row0 + r < n) {
          const float v = f[r][c];
          // M2: position among the sorted levels = number of thresholds strictly below v
          int idx = 0;
#pragma unroll
          for (int s = P >> 1; s >= 1; s >>= 1) idx += (v > tau[idx + s - 1]) ? s : 0;
#pragma unroll
          for (int w = 0; w < NW; ++w) sp[w] = spread[w][idx];
          sx32 = __fadd_rn(sx32, v);
#pragma unroll
          for (int p = 0; p < K; ++p) {
            const int msk = __builtin_amdgcn_sbfe(int(sp[p / 4]), 8 * (p % 4), 1);  // 0 or -1
            a32[p] = __fadd_rn(a32[p], u32_as_f32(f32_as_u32(v) & uint32_t(msk)));
          }
        }
        // M3: row r of the group lands at bit 7-r of each plane byte
#pragma unroll
        for (int w = 0; w < NW; ++w) acc[c][w] = (acc[c][w] << 1) | sp[w];
      }
      Sx += double(sx32);
#pragma unroll
      for (int p = 0; p < K; ++p) A[p] += double(a32[p]);
    }
    // plane bytes of all VEC columns, plane-major, for the counts
    constexpr int CW = (VEC + 3) / 4;
    uint32_t pw[K][CW];
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
        for (int w = 0; w < CW; ++w) cnt[p] += __popc(pw[p][w]);
#pragma unroll
        for (int q = p + 1; q < K; ++q) {
#pragma unroll
          for (int w = 0; w < CW; ++w) dis[pi] += __popc(pw[p][w] ^ pw[q][w]);
          ++pi;
        }
      }
    }
    // payload: byte ((g*m + j)*K + p); the item's VEC*K bytes are contiguous
    uint8_t* dst = payload + ((pos.g * m + pos.jv * VEC) * K);
    if constexpr (VEC > 1) {
      Dwords<NDW> out;
#pragma unroll
      for (int w = 0; w < NDW; ++w) out.v[w] = 0;
#pragma unroll
      for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int p = 0; p < K; ++p) {
          const int b = c * K + p;
          out.v[b / 4] |= ((acc[c][p / 4] >> (8 * (p % 4))) & 0xFFu) << (8 * (b % 4));
        }
      *reinterpret_cast<Dwords<NDW>*>(dst) = out;
    } else {
#pragma unroll
      for (int p = 0; p < K; ++p) dst[p] = uint8_t(acc[0][p / 4] >> (8 * (p % 4)));
    }
  }

  // M4: workgroup totals in a fixed order -> one record per workgroup, stat-major
  double st[NSTAT];
#pragma unroll
  for (int p = 0; p < K; ++p) st[p] = A[p];
  st[K] = Sx;
#pragma unroll
  for (int p = 0; p < K; ++p) st[K + 1 + p] = double(cnt[p]);
#pragma unroll
  for (int i = 0; i < NPAIR; ++i) st[2 * K + 1 + i] = double(dis[i]);
#pragma unroll
  for (int s = 0; s < NSTAT; ++s) {
    const double w = wave_sum(st[s]);
    if ((tid & (kWave - 1)) == 0) red[tid / kWave][s] = w;
  }
  __syncthreads();
  if (tid < NSTAT) {
    double t = red[0][tid];
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) t += red[w][tid];
    partials[int64_t(tid) * gridDim.x + blockIdx.x] = t;
  }
}

// ========================================================================= finalize (M5)
// One workgroup: fixed-order float64 totals, alpha_cur = (B^T B)^-1 B^T x by Gaussian
// elimination with partial pivoting, moving average with beta = min(0.9, (1+t)/(10+t)),
// m_q = mean(B alpha_t - x); header = [alpha_t, m_q].
__global__ __launch_bounds__(kBlock) void mbq_finalize_kernel(const double* __restrict__ partials, int nrec, int k,
                                                               const float* __restrict__ alpha_prev, double n_elems,
                                                               double t, float* __restrict__ header) {
  __shared__ double red[kBlock];
  __shared__ double tot[nstat_of(8)];
  const int tid = threadIdx.x;
  const int nstat = nstat_of(k);
  for (int s = 0; s < nstat; ++s) {
    double a = 0.0;
    for (int b = tid; b < nrec; b += kBlock) a += partials[int64_t(s) * nrec + b];
    red[tid] = a;
    __syncthreads();
    for (int off = kBlock / 2; off > 0; off >>= 1) {
      if (tid < off) red[tid] += red[tid + off];
      __syncthreads();
    }
    if (tid == 0) tot[s] = red[0];
    __syncthreads();
  }
  if (tid != 0) return;
  double G[8][8], h[8], Sb[8], a_prev[8], cur[8];
  const double Sx = tot[k];
  int pi = 0;
  for (int p = 0; p < k; ++p) {
    a_prev[p] = double(alpha_prev[p]);
    h[p] = 2.0 * tot[p] - Sx;                 // B^T x = 2 * (sum over +1 entries) - sum(x)
    Sb[p] = 2.0 * tot[k + 1 + p] - n_elems;   // 1^T B
    G[p][p] = n_elems;
    for (int q = p + 1; q < k; ++q) {
      G[p][q] = G[q][p] = n_elems - 2.0 * tot[2 * k + 1 + pi];
      ++pi;
    }
  }
  double b[8];
  for (int p = 0; p < k; ++p) b[p] = h[p];
  bool singular = false;
  for (int col = 0; col < k && !singular; ++col) {
    int piv = col;
    double best = fabs(G[col][col]);
    for (int r = col + 1; r < k; ++r)
      if (fabs(G[r][col]) > best) { best = fabs(G[r][col]); piv = r; }
    if (best < 1e-9 * n_elems) { singular = true; break; }
    if (piv != col) {
      for (int c = 0; c < k; ++c) { const double tmp = G[col][c]; G[col][c] = G[piv][c]; G[piv][c] = tmp; }
      const double tb = b[col]; b[col] = b[piv]; b[piv] = tb;
    }
    for (int r = col + 1; r < k; ++r) {
      const double fct = G[r][col] / G[col][col];
      for (int c = col; c < k; ++c) G[r][c] -= fct * G[col][c];
      b[r] -= fct * b[col];
    }
  }
  if (singular) {
    for (int p = 0; p < k; ++p) cur[p] = a_prev[p];
  } else {
    for (int r = k - 1; r >= 0; --r) {
      double acc = b[r];
      for (int c = r + 1; c < k; ++c) acc -= G[r][c] * cur[c];
      cur[r] = acc / G[r][r];
    }
  }
  double beta = (1.0 + t) / (10.0 + t);
  if (beta > 0.9) beta = 0.9;
  double dot = 0.0;
  for (int p = 0; p < k; ++p) {
    const float a_t = float(beta * a_prev[p] + (1.0 - beta) * cur[p]);
    header[p] = a_t;
    dot += double(a_t) * Sb[p];
  }
  header[k] = float((dot - Sx) / n_elems);
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
                     partials, d.n, d.m, ipg, p.items, step_for(p.grid, ipg));
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
  p.grid = grid_for(p.items, kEncodeGridMax);
  p.nstat = nstat_of(d.bits);
  // records of the encode kernel (stat-major, kEncodeGridMax wide at most) and, for the
  // residue initialisation, kInitGrid partial sums: both fit the same area
  size_t bytes = size_t(nstat_of(8)) * kEncodeGridMax * sizeof(double);
  p.bytes = (bytes + 255) / 256 * 256;
  return p;
}

hipError_t launch_mbq_compress(const accept_desc& d, const MPlan& p, const void* x, const float* alpha_prev,
                               void* header, void* payload, void* ws, hipStream_t s, StageTimer* tm) {
  double* partials = static_cast<double*>(ws);
  uint8_t* pl = static_cast<uint8_t*>(payload);
  hipError_t e;
  mark(tm, s);
  if (d.in_dtype == ACCEPT_BF16) {
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
  hipLaunchKernelGGL(mbq_finalize_kernel, dim3(1), dim3(kBlock), 0, s, partials, p.grid, d.bits, alpha_prev,
                     double(d.n) * double(d.m), double(d.t), static_cast<float*>(header));
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
  if (d.out_dtype == ACCEPT_BF16) {
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
