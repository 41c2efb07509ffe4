// CPU oracle for the binary-codebook linear layer  y = W_hat . x
//
// TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the
// benchmark's cpu_baseline leg may build, load or call this file.  It shares
// no source, header, table or helper with the HIP library and is deliberately
// plain and slow: no blocking, no fusion, no lookup tables, fp64 throughout.
//
// What it computes (paper: Algorithm "Binary Transformation and Compression",
// steps "Reconstruct binary" and "Dequantize"; appendix "Binary Codebook
// LUT-GEMM", the blockwise definition of W and of y_r):
//
//   idx[i][j]        = bits [j*b, (j+1)*b) of row i's index stream,
//                      b = ceil(log2 K); bit p of a row lives in bit (p & 31)
//                      of that row's 32-bit word (p >> 5)           (integers)
//   B_hat[i][j*v+t]  = +1 if bit t of codebook[idx[i][j]] is set, else -1
//                      (bit = (B+1)/2, the sign<->bit map of Algorithm
//                      "Efficient Binary Vector Packing and Unpacking")
//   W_hat[i][k]      = alpha[i] * B_hat[i][k] + mu[i],   k < in
//   y[m][i]          = sum_{k < in} W_hat[i][k] * x[m][k]      (Y = X W^T)
//
// The paper's two-stage lookup scheme reaches exactly this blockwise dot
// product by re-association, so the oracle is the definition written out.
// The weight matrix is materialised as an fp64 array before it is multiplied.
// Columns k >= in do not exist: surplus positions of the last chunk's pattern
// are never touched.
//
// Also here: the online activation transform that sits in front of the layer
// at inference (section "Learnable Transformation"): X <- X T, T = D P with
// D = diag(sigma), sigma_k = +-1, and P = P1 (x) P2 a Kronecker product.  It
// is written out as the definition too: the n x n matrix T is formed entry by
// entry and the activation row multiplied with it (pins: tests/test_transform_pins.py).
//
// Also here: min-max quantisation of the activations to 8 or 4 bits (section "Activation
// Quantization on sub-bit LLMs", appendix hyper-parameters: min-max quantisation with a scale per
// channel), read as one (offset, step) pair per activation row -- a scale that varied along the
// contraction index could not be taken out of the integer sum -- and the layer on the dequantised
// activations (pins: tests/test_actquant_pins.py).
//
// Also here: the storage variant with several (alpha, mu) groups per weight row
// (btc_oracle_materialise_groups; pins: tests/test_groups_pins.py).
//
// Pins (tests/test_oracle_pins.py): brute force from a byte view of the
// stream, full-codebook dense sign matrix, ones vector -> popcount integers,
// linearity, affine split in (alpha, mu), XNOR-popcount closed form for +-1
// activations, the paper's two-stage table identity, storage accounting,
// fp16/bf16 widening against numpy.
#include <cstdint>
#include <cstring>

extern "C" {

// ceil(log2 K) for K >= 2 (Compression Analysis: ceil(log2 c) bits per vector)
int btc_oracle_index_bits(int K) {
  int b = 0;
  while ((1L << b) < (long)K) ++b;
  return b;
}

long btc_oracle_num_chunks(long in, int v) { return (in + v - 1) / v; }

long btc_oracle_words_per_row(long in, int v, int K) {
  long nbits = btc_oracle_num_chunks(in, v) * (long)btc_oracle_index_bits(K);
  return (nbits + 31) / 32;
}

// Total storage in bits of one layer: v*c for the codebook plus
// ceil(log2 c) * (number of chunks) for the indices (Compression Analysis),
// with chunks counted per row, ceil(in / v) of them.
long btc_oracle_storage_bits(long out, long in, int v, int K) {
  return (long)v * K + (long)btc_oracle_index_bits(K) * out * btc_oracle_num_chunks(in, v);
}

// Index matrix -> per-row LSB-first bit stream, one bit at a time.
// Returns 0, or -1 if some index is outside [0, K).
int btc_oracle_pack(const int32_t* idx, long out, long nchunks, int K, uint32_t* packed) {
  const int b = btc_oracle_index_bits(K);
  const long wpr = (nchunks * b + 31) / 32;
  for (long i = 0; i < out; ++i)
    for (long j = 0; j < nchunks; ++j)
      if (idx[i * nchunks + j] < 0 || idx[i * nchunks + j] >= K) return -1;
  std::memset(packed, 0, sizeof(uint32_t) * (size_t)out * (size_t)wpr);
#pragma omp parallel for schedule(static)
  for (long i = 0; i < out; ++i) {
    uint32_t* row = packed + i * wpr;
    for (long j = 0; j < nchunks; ++j) {
      const uint32_t code = (uint32_t)idx[i * nchunks + j];
      for (int q = 0; q < b; ++q) {
        const long p = j * b + q;
        if ((code >> q) & 1u) row[p >> 5] |= (1u << (p & 31));
      }
    }
  }
  return 0;
}

// Bit stream -> index matrix, one bit at a time.
void btc_oracle_unpack(const uint32_t* packed, long out, long nchunks, int K, int32_t* idx) {
  const int b = btc_oracle_index_bits(K);
  const long wpr = (nchunks * b + 31) / 32;
#pragma omp parallel for schedule(static)
  for (long i = 0; i < out; ++i) {
    const uint32_t* row = packed + i * wpr;
    for (long j = 0; j < nchunks; ++j) {
      uint32_t code = 0;
      for (int q = 0; q < b; ++q) {
        const long p = j * b + q;
        code |= ((row[p >> 5] >> (p & 31)) & 1u) << q;
      }
      idx[i * nchunks + j] = (int32_t)code;
    }
  }
}

// IEEE binary16 bit pattern -> double, exactly.
double btc_oracle_f16_to_f64(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int e = (h >> 10) & 0x1F;
  const int m = h & 0x3FF;
  double val;
  if (e == 0) {
    val = (double)m * (1.0 / 16777216.0);  // m * 2^-24 (zero and subnormals)
  } else if (e == 31) {
    val = m ? __builtin_nan("") : __builtin_inf();
  } else {
    val = (1.0 + (double)m / 1024.0);
    int k = e - 15;
    while (k > 0) { val *= 2.0; --k; }
    while (k < 0) { val *= 0.5; ++k; }
  }
  return sign ? -val : val;
}

// bfloat16 bit pattern -> double, exactly (a bfloat16 is the top half of a float).
double btc_oracle_bf16_to_f64(uint16_t h) {
  const uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return (double)f;
}

// Widen an activation block to fp64.  kind: 0 = fp16, 1 = bf16.
void btc_oracle_widen(const uint16_t* x, long n, int kind, double* xd) {
  for (long t = 0; t < n; ++t)
    xd[t] = kind == 0 ? btc_oracle_f16_to_f64(x[t]) : btc_oracle_bf16_to_f64(x[t]);
}

// Materialise W_hat rows in fp64.  rows == nullptr: all rows 0..out-1 (then
// nrows must equal out); otherwise the listed rows, in the listed order.
// W[r][k] for r < nrows, k < in, row stride `in`.
void btc_oracle_materialise(const uint32_t* packed, const uint32_t* codebook,
                            const float* alpha, const float* mu,
                            long out, long in, int v, int K,
                            const long* rows, long nrows, double* W) {
  (void)out;
  const int b = btc_oracle_index_bits(K);
  const long nchunks = btc_oracle_num_chunks(in, v);
  const long wpr = (nchunks * b + 31) / 32;
#pragma omp parallel for schedule(static)
  for (long r = 0; r < nrows; ++r) {
    const long i = rows ? rows[r] : r;
    const uint32_t* row = packed + i * wpr;
    const double a = (double)alpha[i];
    const double m = (double)mu[i];
    for (long j = 0; j < nchunks; ++j) {
      uint32_t code = 0;
      for (int q = 0; q < b; ++q) {
        const long p = j * b + q;
        code |= ((row[p >> 5] >> (p & 31)) & 1u) << q;
      }
      const uint32_t pattern = codebook[code];
      for (int t = 0; t < v; ++t) {
        const long k = j * v + t;
        if (k >= in) break;
        const double sgn = ((pattern >> t) & 1u) ? 1.0 : -1.0;
        W[r * in + k] = a * sgn + m;
      }
    }
  }
}

// The storage variant with several (alpha, mu) pairs per weight row (Table "Study of Number of Split
// Points"; appendix hyper-parameters: 2 split points by default): the weights of a row are partitioned
// into G groups, every group has its own scale and mean,
//   W_hat[i][k] = alpha[i][g] * B_hat[i][k] + mu[i][g],   g = group[i][k] in [0, G).
// The paper does not print a storage format for the partition; here it is an explicit map of 2 bits per
// weight, row-major, LSB-first like the index stream: group of weight k of row i = bits [2k, 2k+2) of row
// i's map, gwpr = ceil(2 in / 32) words per row.  alpha and mu are [out][G] row-major.  Same calling
// convention as btc_oracle_materialise.
void btc_oracle_materialise_groups(const uint32_t* packed, const uint32_t* codebook,
                                   const float* alpha, const float* mu, const uint32_t* gmap, int G,
                                   long out, long in, int v, int K,
                                   const long* rows, long nrows, double* W) {
  (void)out;
  const int b = btc_oracle_index_bits(K);
  const long nchunks = btc_oracle_num_chunks(in, v);
  const long wpr = (nchunks * b + 31) / 32;
  const long gwpr = (2 * in + 31) / 32;
#pragma omp parallel for schedule(static)
  for (long r = 0; r < nrows; ++r) {
    const long i = rows ? rows[r] : r;
    const uint32_t* row = packed + i * wpr;
    const uint32_t* grow = gmap + i * gwpr;
    for (long j = 0; j < nchunks; ++j) {
      uint32_t code = 0;
      for (int q = 0; q < b; ++q) {
        const long p = j * b + q;                                  // bit q of index j, LSB-first stream
        const uint32_t bit = (row[p / 32] >> (p % 32)) & 1u;
        code += bit << q;
      }
      const uint32_t pattern = codebook[code];
      for (int t = 0; t < v; ++t) {
        const long k = j * v + t;
        if (k >= in) break;
        const int g = (int)((grow[(2 * k) >> 5] >> ((2 * k) & 31)) & 3u);
        const double sgn = (pattern & (1u << t)) != 0u ? 1.0 : -1.0;   // bit t set: +1
        W[r * in + k] = (double)alpha[i * G + g] * sgn + (double)mu[i * G + g];
      }
    }
  }
}

// Y[m][r] = sum_k W[r][k] * X[m][k], k ascending, fp64.  X is fp64 [M][in],
// W is [nrows][in], Y is [M][nrows].
void btc_oracle_matmul(const double* W, long nrows, long in,
                       const double* X, long M, double* Y) {
#pragma omp parallel for schedule(static)
  for (long r = 0; r < nrows; ++r) {
    const double* w = W + r * in;
    for (long m = 0; m < M; ++m) {
      const double* x = X + m * in;
      double acc = 0.0;
      for (long k = 0; k < in; ++k) acc += w[k] * x[k];
      Y[m * nrows + r] = acc;
    }
  }
}

// Online activation transform, section "Learnable Transformation" (transformation
// pair T = D P, P = P1 (x) P2) and "Integration into Transformer Architecture"
// (X <- X T):
//   T[i][j] = sigma_i * P1[i1][j1] * P2[i2][j2],  i = i1*n2 + i2,  j = j1*n2 + j2
//   Y[m][j] = sum_i X[m][i] * T[i][j]
// sigma_i = +1 where bit (i & 31) of sign_bits[i >> 5] is set, else -1 (the
// same sign<->bit map as the codebook).  X is fp64 [M][n] (already widened),
// P1 is fp32 [n1][n1], P2 is fp32 [n2][n2], both row-major; Y fp64 [M][n].
// T is formed one column at a time (n doubles), never blocked or factored.
void btc_oracle_transform(const double* X, long M, long n1, long n2, const uint32_t* sign_bits,
                          const float* P1, const float* P2, double* Y) {
  const long n = n1 * n2;
#pragma omp parallel for schedule(static)
  for (long j = 0; j < n; ++j) {
    const long j1 = j / n2, j2 = j % n2;
    double* col = new double[n];
    for (long i = 0; i < n; ++i) {
      const long i1 = i / n2, i2 = i % n2;
      const double sigma = ((sign_bits[i >> 5] >> (i & 31)) & 1u) ? 1.0 : -1.0;
      col[i] = sigma * ((double)P1[i1 * n1 + j1] * (double)P2[i2 * n2 + j2]);
    }
    for (long m = 0; m < M; ++m) {
      const double* x = X + m * n;
      double acc = 0.0;
      for (long i = 0; i < n; ++i) acc += x[i] * col[i];
      Y[m * n + j] = acc;
    }
    delete[] col;
  }
}

// E-step of the binary codebook clustering (section "Binary Codebook Compression", step
// "E-step Assignment"): z_i = argmin_k || b_i - c_k ||_2^2 over +-1 vectors of length v, a vector
// identical to a centroid being assigned to it (distance 0 is the minimum, so the rule is the
// argmin itself).  Written from the definition: elements are expanded to +-1 integers and the
// squared differences are summed.  Among equally near centroids the lowest index wins (the paper
// leaves ties open).  Bit t of a pattern is element t (set => +1); bits >= v are ignored.
// dist2[i] receives the squared distance to the chosen centroid (may be null).
void btc_oracle_assign(const uint32_t* vectors, long N, int v, const uint32_t* codebook, long K,
                       int32_t* z, int32_t* dist2) {
#pragma omp parallel for schedule(static)
  for (long i = 0; i < N; ++i) {
    long best_k = -1;
    int best = 0;
    for (long k = 0; k < K; ++k) {
      int d2 = 0;
      for (int t = 0; t < v; ++t) {
        const int b = ((vectors[i] >> t) & 1u) ? 1 : -1;
        const int c = ((codebook[k] >> t) & 1u) ? 1 : -1;
        d2 += (b - c) * (b - c);
      }
      if (best_k < 0 || d2 < best) {
        best = d2;
        best_k = k;
      }
    }
    z[i] = (int32_t)best_k;
    if (dist2) dist2[i] = best;
  }
}

// M-step of the binary codebook clustering (section "Flash and Accurate Binary Codebook", step
// "M-step Centroid Update"; the loop over clusters in the algorithm of appendix "Binary Codebook
// Optimization"): for every cluster k with at least one assigned vector, the centroid becomes the
// sign of the dimension-wise mean of its vectors, a zero mean giving +1; an empty cluster keeps its
// centroid.  Written from the definition: the +-1 elements are summed as integers per cluster and
// dimension.  Bits >= v of a new centroid are zero; an unchanged centroid is left as it was.
// z[i] outside [0, K) is an error (returns -1, nothing written).
int btc_oracle_update(const uint32_t* vectors, const int32_t* z, long N, int v, uint32_t* codebook, long K) {
  for (long i = 0; i < N; ++i)
    if (z[i] < 0 || z[i] >= K) return -1;
  for (long k = 0; k < K; ++k) {
    long size = 0;
    long sum[32] = {0};
    for (long i = 0; i < N; ++i) {
      if (z[i] != k) continue;
      ++size;
      for (int t = 0; t < v; ++t) sum[t] += ((vectors[i] >> t) & 1u) ? 1 : -1;
    }
    if (size == 0) continue;
    uint32_t c = 0;
    for (int t = 0; t < v; ++t)
      if (sum[t] >= 0) c |= 1u << t;           // sign(mean), sign(0) = +1
    codebook[k] = c;
  }
  return 0;
}

// Min-max quantisation of activation rows to `bits` bits (section "Activation Quantization on sub-bit
// LLMs"; appendix: min-max quantisation, one scale per channel -- here: per activation row):
//   lo[m]   = min_k x[m][k],  hi = max_k x[m][k]
//   step[m] = (hi - lo) / (2^bits - 1)            (1 if the row is constant)
//   q[m][k] = round_half_even((x[m][k] - lo[m]) / step[m])  clamped to [0, 2^bits - 1]
//   x ~ lo[m] + step[m] * q[m][k]
// The integer q is decided by floating-point arithmetic, so the precision is part of the definition:
// every operation above is a single IEEE fp32 operation in the order written (x widened exactly).
void btc_oracle_quantize_rows(const float* X, long M, long n, int bits, int32_t* q, float* lo, float* step) {
  const float levels = (float)((1 << bits) - 1);
#pragma omp parallel for schedule(static)
  for (long m = 0; m < M; ++m) {
    const float* x = X + m * n;
    float mn = x[0], mx = x[0];
    for (long k = 1; k < n; ++k) {
      if (x[k] < mn) mn = x[k];
      if (x[k] > mx) mx = x[k];
    }
    const float range = mx - mn;
    const float st = range > 0.0f ? range / levels : 1.0f;
    lo[m] = mn;
    step[m] = st;
    for (long k = 0; k < n; ++k) {
      const float t = x[k] - mn;
      const float r = __builtin_nearbyintf(t / st);     // round to nearest, ties to even
      q[m * n + k] = r < 0.0f ? 0 : (r > levels ? (int32_t)levels : (int32_t)r);
    }
  }
}

}  // extern "C"
