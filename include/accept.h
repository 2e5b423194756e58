/*
 * accept.h -- C ABI of the MI355X (gfx950) bit-level compressor / decompressor for the
 * activations and gradients that cross a pipeline-partition boundary.
 *
 * The operations are those of the paper's sections "Bit-level Fast Compression Scheme"
 * and "Bit-level Fast Decompression Scheme":
 *
 *   scheme ACCEPT_UNIFORM ("backward", gradients): c = max|g|, s = c/(2^(k-1)-1), round
 *     g/s to a k-bit signed integer, offset to unsigned and concatenate the codes into
 *     bytes (paragraphs "Backward Quantizer", "Backward Encoder"); the inverse splits the
 *     bytes, removes the offset and multiplies by s ("Backward Decoder", "Backward
 *     Dequantizer").
 *   scheme ACCEPT_MBQ ("forward", features): x ~ B alpha with B in {-1,+1}^(N x k); B is
 *     the nearest of the 2^k values sum(+-alpha_j) of the previous batch's alpha, alpha
 *     is then refreshed by least squares and a moving average (eqs. (MBQ), (alpha
 *     solution), (alpha update)), the mean quantization error is sent along (eq. (biased
 *     error)), and the sign bits are packed eight batch entries to a byte, one bit plane
 *     per basis (paragraph "Forward Encoder"); the inverse is "Forward Decoder" and
 *     "Forward Dequantizer" (x_hat = B alpha - m_q).
 *
 * A tensor is given as (n, m): n is the leading ("batch") dimension, m the product of the
 * others, N = n*m elements in row-major order.
 *
 * Memory: every pointer named *_dev is DEVICE memory of the current HIP device; the
 * descriptor and the size outputs are HOST memory.  The caller allocates and owns all
 * buffers; the library allocates no device memory, keeps no state between calls (what a
 * later call needs stays in the caller's workspace), enqueues its kernels on the given stream
 * and returns without waiting for them.  The measurement entry points that bracket kernels
 * with events and wait are declared apart, in accept_profile.h.
 *
 * Errors: every function returns an accept_status; nothing is thrown across the ABI.
 * When a call fails validation, no kernel is launched and no output byte is written.
 * Non-finite inputs are not detected; their codes are unspecified (but stay inside the
 * payload buffer).
 */
#ifndef ACCEPT_H
#define ACCEPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ACCEPT_OK = 0,
  ACCEPT_ERR_INVALID_ARG = 1,      /* null pointer, bad size, bits out of range, misaligned buffer */
  ACCEPT_ERR_UNSUPPORTED = 2,      /* valid, but beyond a fixed limit of the entry point called  */
  ACCEPT_ERR_BUFFER_TOO_SMALL = 3, /* never returned by the C functions (they take no capacities);
                                      the Python binding raises it for a tensor that is smaller
                                      than accept_packed_size / accept_workspace_size require  */
  ACCEPT_ERR_HIP = 4               /* a HIP runtime call or kernel launch failed              */
} accept_status;

enum { ACCEPT_UNIFORM = 0, ACCEPT_MBQ = 1 };      /* accept_desc.scheme                     */
enum { ACCEPT_F32 = 0, ACCEPT_BF16 = 1 };         /* accept_desc.in_dtype / out_dtype       */
enum { ACCEPT_ROUND_NEAREST_EVEN = 0, ACCEPT_ROUND_STOCHASTIC = 1 }; /* accept_desc.rounding */
/* accept_desc.layout: how the integers are laid into the payload.
 *   PACKED     the forms this library is built around: UNIFORM a dense stream of k-bit codes
 *              in flat element order, MBQ bit planes along the batch dimension.
 *   BATCH      UNIFORM only, k in {2, 4, 8}: the layout of the paper's "Backward Encoder",
 *              where the shifted codes of 8/k consecutive batch entries of one column share
 *              a byte (byte g*m + j holds rows g*(8/k) .. of column j, first row in the most
 *              significant bits, rows >= n as 0 bits); ceil(n/(8/k))*m bytes.
 *   UNENCODED  the "w/o enc." rows of the paper's size table: every transmitted integer in
 *              a byte of its own.  UNIFORM: q as a two's-complement byte, n*m bytes.  MBQ:
 *              each binary base as +1 / -1, element-major with the k bases innermost,
 *              n*m*k bytes.
 * BATCH and UNENCODED exist to measure what the packed layouts buy; their kernels are plain. */
enum { ACCEPT_LAYOUT_PACKED = 0, ACCEPT_LAYOUT_BATCH = 1, ACCEPT_LAYOUT_UNENCODED = 2 };

/*
 * Problem descriptor (host memory, plain data, 64 bytes).
 *
 *  scheme    ACCEPT_UNIFORM or ACCEPT_MBQ.
 *  bits      k.  UNIFORM: 2..8 (the paper uses 8 and 4).  MBQ: 1..8 (the paper uses 2..4).
 *  in_dtype  element type of x (compress).  out_dtype: element type of x_hat (decompress).
 *  n, m      tensor geometry, n >= 1, m >= 1, n*m <= 2^40.
 *  channels  UNIFORM only.  0 or 1: one range for the tensor (the paper's rule).  C > 1:
 *            one range per channel, C must divide m and the channel of flat element i is
 *            (i mod m) / (m/C)  (dimension 1 of an n x C x ... tensor).  MBQ: must be 0/1.
 *  rounding  UNIFORM only.  ACCEPT_ROUND_NEAREST_EVEN: round half to even (reproducible
 *            streams).  ACCEPT_ROUND_STOCHASTIC: the paper's rule, floor(v)+1 with
 *            probability v-floor(v); the uniform number of element i is the top 24 bits
 *            of splitmix64's output function at seed + (i+1)*0x9E3779B97F4A7C15.
 *  layout    ACCEPT_LAYOUT_PACKED (0) unless one of the comparison layouts is wanted.
 *  seed      seed of the stochastic rounding.
 *  t         MBQ only: batch index in beta = min(0.9, (1+t)/(10+t))  (eq. (alpha update)).
 */
typedef struct {
  int32_t  scheme;
  int32_t  bits;
  int32_t  in_dtype;
  int32_t  out_dtype;
  int64_t  n;
  int64_t  m;
  int64_t  channels;
  int32_t  rounding;
  int32_t  layout;
  uint64_t seed;
  int64_t  t;
} accept_desc;

/*
 * Sizes of the compressed representation (section "Transmission Data Comparison").
 *   UNIFORM: header = 4*max(channels,1) bytes (float32 scale s per range group),
 *            payload = ceil(N*k/8) bytes.
 *   MBQ:     header = 4*(k+1) bytes (alpha_t[0..k), then m_q), payload = ceil(n/8)*m*k bytes.
 *   Payload of the comparison layouts: see accept_desc.layout.
 * On a wire the two are concatenated header first; the total equals the paper's formulas.
 * Host-only; needs no GPU.
 */
accept_status accept_packed_size(const accept_desc* desc, size_t* header_bytes, size_t* payload_bytes);

/* Bytes of device scratch accept_compress, accept_mbq_init and accept_mbq_compress_first need
 * for this descriptor (host-only; always a multiple of 256; depends on the descriptor alone,
 * not on the device).  See accept_compress for how the workspace is to be prepared. */
accept_status accept_workspace_size(const accept_desc* desc, size_t* bytes);

/*
 * Compress x_dev (N elements of in_dtype, 16-byte aligned) into header_dev (4-byte
 * aligned) and payload_dev (16-byte aligned), sizes as accept_packed_size reports.
 *
 *   UNIFORM: range pass, then fused quantize + pack.  Code i occupies payload bits
 *     [ik, (i+1)k), most significant bit first, bit b of the stream being bit 7-(b mod 8)
 *     of byte b/8; codes are q + 2^(k-1) for k < 8 and the two's-complement byte for
 *     k = 8; unused bits of the last byte are 0.  q = clamp(round(x * fl(L/c)), -2^(k-1), L),
 *     L = 2^(k-1)-1; a range below 2^-100 gives s = 0 and all-zero q.
 *     alpha_prev_dev is ignored (may be null).
 *   MBQ: alpha_prev_dev points at k floats (alpha of the previous batch, or of the
 *     residue initialisation).  One pass assigns every element to its nearest level,
 *     writes the bit planes (byte ((g*m + j)*k + p), g = row/8, holds bit p of rows
 *     8g..8g+7 of column j, first row in the most significant bit, rows >= n as 0) and
 *     accumulates the least-squares sums; a second, small kernel solves for alpha_t
 *     (eqs. (alpha solution), (alpha update)) and writes header = [alpha_t, m_q].  Feed
 *     header[0..k) back as alpha_prev of the next batch.
 *
 * workspace_dev: accept_workspace_size bytes, 256-byte aligned.  Zero-fill it once after
 * allocating it (hipMemset); from then on the library keeps it in the state its next call
 * needs (its first 16 KiB hold counters that every call leaves at zero; the rest is
 * scratch whose contents do not matter), so one workspace serves any number of calls and
 * descriptors of both schemes, one call at a time: calls that share a workspace must not
 * overlap.
 * hip_stream: a hipStream_t (null = the default stream).
 */
accept_status accept_compress(const accept_desc* desc, const void* x_dev, const float* alpha_prev_dev,
                              void* header_dev, void* payload_dev, void* workspace_dev, void* hip_stream);

/*
 * Decompress header_dev + payload_dev into xhat_dev (N elements of out_dtype, 16-byte
 * aligned): UNIFORM x_hat = float(q) * s (one float32 multiply); MBQ x_hat = (sum of
 * +-alpha_p in the order p = 0..k-1 from 0) - m_q.  bfloat16 output is the round-to-
 * nearest-even image of the float32 result.  One kernel, no workspace.
 */
accept_status accept_decompress(const accept_desc* desc, const void* header_dev, const void* payload_dev,
                                void* xhat_dev, void* hip_stream);

/*
 * accept_compress for callers that cannot allocate device memory or own no workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels, outputs and errors as accept_compress, except that the workspace is an
 * array of ACCEPT_NOALLOC_SCRATCH_BYTES that is part of the library's device code: every GPU
 * the library runs on holds its own copy from the first launch until the process ends.  The
 * call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine);
 * its first use on a device looks the array's address up once (hipGetSymbolAddress).
 * Descriptors whose accept_workspace_size exceeds ACCEPT_NOALLOC_SCRATCH_BYTES are rejected
 * with ACCEPT_ERR_UNSUPPORTED before any HIP call (every MBQ descriptor and every per-tensor
 * UNIFORM descriptor fits; per-channel ones fit up to about 250,000 (row, channel) segments).
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 * (different streams or threads) race; calls on one stream are safe.  The array starts
 * zero-filled when the library is loaded and every kernel leaves its counters at zero, which
 * is all the kernels rely on, so no clearing is enqueued.
 */
enum { ACCEPT_NOALLOC_SCRATCH_BYTES = 1 << 20 };
accept_status accept_compress_noalloc(const accept_desc* desc, const void* x_dev, const float* alpha_prev_dev,
                                      void* header_dev, void* payload_dev, void* hip_stream);

/*
 * Residue-based initialisation of alpha at batch 0 of an epoch (paragraph "Forward
 * Quantizer"): alpha_j = mean|rho_j|, rho_0 = x, rho_(j+1) = rho_j - alpha_j sign(rho_j)
 * (sign(0) = +1).  Writes k floats to alpha0_dev.  MBQ descriptors only; workspace as
 * for accept_compress.
 */
accept_status accept_mbq_init(const accept_desc* desc, const void* x_dev, float* alpha0_dev,
                              void* workspace_dev, void* hip_stream);

/*
 * Compression of batch 0 of an epoch (paragraph "Forward Quantizer": at batch 0 B^0 and
 * alpha^0 come from the residue method and are what is sent; the search among the levels of
 * the previous batch starts at batch 1).  Writes payload = the bit planes of B^0 (b_j =
 * sign(rho_j), layout as accept_compress) and header = [alpha^0, m_q] with m_q =
 * mean(B^0 alpha^0 - x) (eq. (biased error)); accept_decompress reads them like any other
 * batch, and header[0..k) is alpha_prev of batch 1.  k passes over x (alpha_j needs the whole
 * tensor's |rho_j|); the last one also writes the planes.  MBQ descriptors with
 * ACCEPT_LAYOUT_PACKED only; desc->t is ignored; buffers and workspace as for accept_compress.
 */
accept_status accept_mbq_compress_first(const accept_desc* desc, const void* x_dev, void* header_dev,
                                        void* payload_dev, void* workspace_dev, void* hip_stream);

/*
 * Adaptive bit width.  direction 0 (forward): 2, then +1 per learning-rate change, at
 * most 4.  direction 1 (backward): 8 until the learning rate first changes, then 4.
 * (Paragraphs after eq. (biased error) and after the stochastic-rounding equation.)
 * Returns -1 for a bad direction or a negative count.  Host-only.
 */
int accept_bits_schedule(int direction, int lr_changes_so_far);

/* Human-readable name of a status code (static storage). */
const char* accept_status_string(accept_status status);

/* Library version, "major.minor.patch" (static storage). */
const char* accept_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ACCEPT_H */
