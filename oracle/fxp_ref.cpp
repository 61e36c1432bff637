// fxp_ref — CPU ORACLE for the integer (dynamic fixed-point) linear-layer step.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
// correct CPU implementation that the GPU library is checked against.  Only the
// test-suite, the smoke check and the benchmark's "cpu_baseline" leg may call
// it.  It shares no source, header, table or helper with the HIP kernels and
// neither side includes or links the other.
//
// Every function follows one passage of "Is Integer Arithmetic Enough for Deep
// Learning Training?" (arXiv 2207.08822) in the paper's own order and notation:
//   scale  — Sec. 3.1: e_max = max(e_1..e_n), the shared per-tensor scale.
//   map    — Sec. 3.1 + App. A.1 (Fig. 4): unpack, shift the 24-bit mantissa
//            right by e_max-e_i, round the result stochastically to 7 bits by
//            comparing a random number with the low 17 bits, attach the sign.
//   gemm   — Sec. 3.3 (Fig. 2): int8 x int8 products accumulated in int32.  An int32 sum holds any
//            contraction of up to 133144 terms (127^2 * 133144 < 2^31).  For longer ones (the weight
//            gradient of a layer applied to more rows than that) the paper gives nothing; this build
//            takes what the int32 sum is an instance of, the exact integer sum, held in int64
//            (gemm64), and the inverse mapping rounds it once (unmap64).
//   unmap  — Sec. 3.2 (Fig. 1b): shared exponent (sum of the operand
//            exponents, Sec. 3.3) + integer mantissa -> rounded, normalised,
//            packed fp32.
//   linear — App. A.2: Y = X W, dL/dW = X^T G, and dL/dX = G W^T (chain rule).
//   conv   — Sec. 3.4: the same inner products with the convolution's index pattern.
//   bmm    — Sec. 5 (vision transformer): the attention products Q K^T and A V, one product per head.
//   sgd16  — Remark 5 + App. A.4: w_hat + alpha_hat * g_hat with int16 mantissas (parity unpinned, below).
// Random numbers: the paper only says they are generated on the fly; this
// build fixes Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), keyed by the
// seed, with the tensor's stream id and the element index as the counter.
//
// Parity pins (tests that do not depend on this file's own formulas) exist for
// every function: the paper's two worked examples, exact round trips, an exact
// rational model, numpy int64 matmul, an integer round-to-nearest-even model,
// 10^7-sample mean-error and closed-form variance tests, and, for the Philox
// rounds, rocRAND's host-callable engine (an independent implementation of the
// same published generator; the authors' known-answer vectors themselves are
// not available offline).
// PARITY UNPINNED: axpy16 / sgd16.  The paper states the integer update only as w_hat + alpha_hat * g_hat with
// stochastic rounding (App. A.4) and gives neither the alignment of the two terms nor the place of the
// rounding; the formula below is this build's reading.  Its tests check what the paper does fix (the operands
// are the int16 instance of the map; the update is unbiased; representable operands give the exact result) but
// cannot show that another reading was not meant.
//
// Build: g++ -O2 -fopenmp -shared -fPIC (see oracle/build.py).  OpenMP only
// splits independent outer loops; results do not depend on the thread count.

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---- unpack (Sec. 3.1, "unpack to integer") --------------------------------
struct Unpacked {
    uint32_t s;  // sign bit
    uint32_t e;  // 8-bit exponent field
    uint32_t f;  // 23-bit fraction field
};

Unpacked unpack(float x) {
    uint32_t b;
    std::memcpy(&b, &x, sizeof b);
    Unpacked u;
    u.s = b >> 31;
    u.e = (b >> 23) & 0xFFu;
    u.f = b & 0x7FFFFFu;
    return u;
}

// A sub-normal input (e == 0) has no hidden bit and weighs as much as e == 1.
uint32_t effective_exponent(const Unpacked& u) { return u.e == 0 ? 1u : u.e; }

// 24-bit mantissa: the 23 fraction bits plus the implicit hidden bit.
uint32_t mantissa24(const Unpacked& u) { return (u.e == 0 ? 0u : 0x800000u) | u.f; }

// ---- Philox-4x32-10 ---------------------------------------------------------
void mulhilo(uint32_t a, uint32_t b, uint32_t& hi, uint32_t& lo) {
    const uint64_t p = static_cast<uint64_t>(a) * static_cast<uint64_t>(b);
    hi = static_cast<uint32_t>(p >> 32);
    lo = static_cast<uint32_t>(p);
}

void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
    const uint32_t MUL0 = 0xD2511F53u, MUL1 = 0xCD9E8D57u;   // round multipliers
    const uint32_t WEYL0 = 0x9E3779B9u, WEYL1 = 0xBB67AE85u; // key increments
    uint32_t c[4] = {ctr_in[0], ctr_in[1], ctr_in[2], ctr_in[3]};
    uint32_t k[2] = {key_in[0], key_in[1]};
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k[0] += WEYL0;
            k[1] += WEYL1;
        }
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo(MUL0, c[0], hi0, lo0);
        mulhilo(MUL1, c[2], hi1, lo1);
        const uint32_t n0 = hi1 ^ c[1] ^ k[0];
        const uint32_t n1 = lo1;
        const uint32_t n2 = hi0 ^ c[3] ^ k[1];
        const uint32_t n3 = lo0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

// The 32-bit random word of element i of tensor-stream `stream_id`:
// counter = (i/4 as 64 bits, stream_id as 64 bits), key = seed, word i mod 4.
uint32_t random_word(uint64_t seed, uint64_t stream_id, uint64_t i) {
    const uint64_t block = i >> 2;
    const uint32_t ctr[4] = {static_cast<uint32_t>(block), static_cast<uint32_t>(block >> 32),
                             static_cast<uint32_t>(stream_id), static_cast<uint32_t>(stream_id >> 32)};
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return out[i & 3u];
}

// ---- map of one element (Sec. 3.1, App. A.1) --------------------------------
// bits = total width of the fixed-point value (sign + bits-1 magnitude bits);
// the paper's int8 is bits = 8: 24-bit mantissa rounded to 7 bits using the
// low 17 bits.  rounding 0 = stochastic, 1 = nearest (half up on magnitude).
int32_t map_one(float x, int32_t e_max, uint32_t word, int rounding, int bits) {
    const Unpacked u = unpack(x);
    const int mag_bits = bits - 1;
    const int cut = 24 - mag_bits;                   // number of low bits dropped
    const uint32_t sat = (1u << mag_bits) - 1u;      // largest magnitude
    uint32_t q1;
    if (u.e == 255u) {
        // not a number the format can carry: Inf saturates, NaN gives 0
        q1 = (u.f == 0u) ? sat : 0u;
    } else {
        const int32_t d = e_max - static_cast<int32_t>(effective_exponent(u));
        if (d < 0) {
            q1 = sat;                                // above the range of this scale
        } else {
            const uint32_t m = mantissa24(u);
            const uint32_t m_shift = (d >= 24) ? 0u : (m >> d);  // truncating right shift
            const uint32_t q0 = m_shift >> cut;                  // bits kept
            const uint32_t low = m_shift & ((1u << cut) - 1u);   // bits dropped
            if (rounding == 0) {
                const uint32_t r = word >> (32 - cut);           // uniform on [0, 2^cut)
                q1 = q0 + ((r < low) ? 1u : 0u);                 // P(up) = low / 2^cut
            } else {
                q1 = (m_shift + (1u << (cut - 1))) >> cut;
            }
            if (q1 > sat) q1 = sat;
        }
    }
    return u.s ? -static_cast<int32_t>(q1) : static_cast<int32_t>(q1);
}

// exponent of one unit of a mapped tensor: value = q * 2^lsb_exponent
int32_t lsb_exponent(int32_t e_max, int bits) { return e_max - 127 - (bits - 2); }

bool bad_bits(int bits) { return bits < 2 || bits > 8; }

}  // namespace

extern "C" {

int fxp_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void fxp_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    philox4x32_10(ctr, key, out);
}

uint32_t fxp_ref_random_word(uint64_t seed, uint64_t stream_id, uint64_t i) {
    return random_word(seed, stream_id, i);
}

// Sec. 3.1: e_max = max_i e_i (sub-normals and zeros count as e = 1).
int fxp_ref_scale(const float* x, uint64_t n, int32_t* e_max) {
    if (!e_max || (n && !x)) return -1;
    int32_t best = 1;
#pragma omp parallel for reduction(max : best) schedule(static)
    for (int64_t i = 0; i < static_cast<int64_t>(n); ++i) {
        const int32_t e = static_cast<int32_t>(effective_exponent(unpack(x[i])));
        if (e > best) best = e;
    }
    *e_max = best;
    return 0;
}

// Sec. 3.1 + App. A.1: x[rows, cols] row-major -> q[rows, cols] (and, when qT
// is given, the same values transposed to [cols, rows]).
int fxp_ref_map(const float* x, int64_t rows, int64_t cols, int32_t e_max, int8_t* q, int8_t* qT,
                uint64_t seed, uint64_t stream_id, int rounding, int bits) {
    if (rows < 0 || cols < 0 || bad_bits(bits) || rounding < 0 || rounding > 1) return -2;
    if (rows * cols > 0 && (!x || (!q && !qT))) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            const uint64_t i = static_cast<uint64_t>(r) * static_cast<uint64_t>(cols) + static_cast<uint64_t>(c);
            const uint32_t word = random_word(seed, stream_id, i);
            const int8_t v = static_cast<int8_t>(map_one(x[i], e_max, word, rounding, bits));
            if (q) q[i] = v;
            if (qT) qT[c * rows + r] = v;
        }
    }
    return 0;
}

// The same for `nrows` consecutive rows of a larger [*, cols] tensor, starting at row `row0`: x and q hold only
// those rows, the random word of an element is the one of its index in the whole tensor, (row0 + r) * cols + c.
// Lets a test check slices of a tensor too large to map whole on the CPU.
int fxp_ref_map_rows(const float* x, int64_t row0, int64_t nrows, int64_t cols, int32_t e_max, int8_t* q, uint64_t seed,
                     uint64_t stream_id, int rounding, int bits) {
    if (row0 < 0 || nrows < 0 || cols < 0 || bad_bits(bits) || rounding < 0 || rounding > 1) return -2;
    if (nrows * cols > 0 && (!x || !q)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            const uint64_t local = static_cast<uint64_t>(r) * static_cast<uint64_t>(cols) + static_cast<uint64_t>(c);
            const uint64_t i = static_cast<uint64_t>(row0 + r) * static_cast<uint64_t>(cols) + static_cast<uint64_t>(c);
            q[local] = static_cast<int8_t>(map_one(x[local], e_max, random_word(seed, stream_id, i), rounding, bits));
        }
    }
    return 0;
}

// Sec. 3.3: C[M,N] = op(A)[M,K] * op(B)[K,N], int8 operands, int32 accumulation.
// transA = 0: A is stored [M,K] (lda >= K); 1: A is stored [K,M] (lda >= M).
// transB = 0: B is stored [K,N] (ldb >= N); 1: B is stored [N,K] (ldb >= K).
int fxp_ref_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                 const int8_t* B, int64_t ldb, int32_t* C, int64_t ldc) {
    if (M < 0 || N < 0 || K < 0 || ldc < N) return -2;
    if (M * N > 0 && !C) return -1;
    if (M * K > 0 && !A) return -1;
    if (N * K > 0 && !B) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k) {
                const int32_t a = transA ? A[k * lda + i] : A[i * lda + k];
                const int32_t b = transB ? B[j * ldb + k] : B[k * ldb + j];
                acc += a * b;
            }
            C[i * ldc + j] = acc;
        }
    }
    return 0;
}

// Sec. 3.2 + 3.3: the real number acc * 2^E with E = lsb(eA) + lsb(eB), rounded
// once (nearest, ties to even) to fp32.  bitsB == 0 means "no second operand"
// (the inverse map of a mapped tensor itself).
int fxp_ref_unmap(const int32_t* acc, uint64_t n, int32_t eA, int bitsA, int32_t eB, int bitsB, float* out) {
    if (n && (!acc || !out)) return -1;
    if (bad_bits(bitsA) || (bitsB != 0 && bad_bits(bitsB))) return -2;
    const int32_t E = lsb_exponent(eA, bitsA) + (bitsB ? lsb_exponent(eB, bitsB) : 0);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < static_cast<int64_t>(n); ++i) {
        out[i] = static_cast<float>(std::ldexp(static_cast<double>(acc[i]), E));
    }
    return 0;
}

int fxp_ref_unmap_i8(const int8_t* q, uint64_t n, int32_t eA, int bitsA, float* out) {
    if (n && (!q || !out)) return -1;
    if (bad_bits(bitsA)) return -2;
    const int32_t E = lsb_exponent(eA, bitsA);
    for (uint64_t i = 0; i < n; ++i) out[i] = static_cast<float>(std::ldexp(static_cast<double>(q[i]), E));
    return 0;
}

// The longest contraction whose sums an int32 accumulator always holds.
static const int64_t kInt32Terms = 133144;

// The same product with the exact sum held in int64: for contractions beyond kInt32Terms.
int fxp_ref_gemm64(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                   const int8_t* B, int64_t ldb, int64_t* C, int64_t ldc) {
    if (M < 0 || N < 0 || K < 0 || ldc < N) return -2;
    if (M * N > 0 && !C) return -1;
    if (M * K > 0 && !A) return -1;
    if (N * K > 0 && !B) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) {
                const int64_t a = transA ? A[k * lda + i] : A[i * lda + k];
                const int64_t b = transB ? B[j * ldb + k] : B[k * ldb + j];
                acc += a * b;
            }
            C[i * ldc + j] = acc;
        }
    }
    return 0;
}

// Inverse mapping of such a sum: |acc| < 2^53 (127^2 * 2^31 terms at most), so the conversion to double
// and the scaling are exact and the value is rounded once, to fp32.
int fxp_ref_unmap64(const int64_t* acc, uint64_t n, int32_t eA, int bitsA, int32_t eB, int bitsB, float* out) {
    if (n && (!acc || !out)) return -1;
    if (bad_bits(bitsA) || (bitsB != 0 && bad_bits(bitsB))) return -2;
    const int32_t E = lsb_exponent(eA, bitsA) + (bitsB ? lsb_exponent(eB, bitsB) : 0);
    for (int64_t i = 0; i < static_cast<int64_t>(n); ++i) {
        if (acc[i] >= (int64_t{1} << 53) || acc[i] <= -(int64_t{1} << 53)) return -2;
        out[i] = static_cast<float>(std::ldexp(static_cast<double>(acc[i]), E));
    }
    return 0;
}

// product + inverse mapping of a layer: int32 sums where they are sure to fit, int64 sums beyond
static int product_unmap(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                         const int8_t* B, int64_t ldb, int32_t eA, int32_t eB, int bits, float* out) {
    const size_t n = static_cast<size_t>(M * N);
    int rc;
    if (K <= kInt32Terms) {
        int32_t* acc = new int32_t[n + 1];
        rc = fxp_ref_gemm(transA, transB, M, N, K, A, lda, B, ldb, acc, N);
        if (!rc) rc = fxp_ref_unmap(acc, n, eA, bits, eB, bits, out);
        delete[] acc;
    } else {
        int64_t* acc = new int64_t[n + 1];
        rc = fxp_ref_gemm64(transA, transB, M, N, K, A, lda, B, ldb, acc, N);
        if (!rc) rc = fxp_ref_unmap64(acc, n, eA, bits, eB, bits, out);
        delete[] acc;
    }
    return rc;
}

// App. A.2, forward: Y = unmap(map(X) * map(W)).  X[M,K], W[K,N], Y[M,N].
// Xq[M,K], Wq[K,N] and the two scales are returned for the backward pass.
// Random streams: (step << 8) | tag with tag 0 for X and 1 for W.
int fxp_ref_linear_fwd(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y, int8_t* Xq,
                       int8_t* Wq, int32_t* eX, int32_t* eW, uint64_t seed, uint64_t step, int rounding, int bits) {
    if (!X || !W || !Y || !Xq || !Wq || !eX || !eW) return -1;
    int rc;
    if ((rc = fxp_ref_scale(X, static_cast<uint64_t>(M * K), eX))) return rc;
    if ((rc = fxp_ref_scale(W, static_cast<uint64_t>(K * N), eW))) return rc;
    if ((rc = fxp_ref_map(X, M, K, *eX, Xq, nullptr, seed, (step << 8) | 0u, rounding, bits))) return rc;
    if ((rc = fxp_ref_map(W, K, N, *eW, Wq, nullptr, seed, (step << 8) | 1u, rounding, bits))) return rc;
    return product_unmap(0, 0, M, N, K, Xq, K, Wq, N, *eX, *eW, bits, Y);
}

// App. A.2, backward: G = map(dY) once (stream tag 2); dX = unmap(G * Wq^T)
// [M,K]; dW = unmap(Xq^T * G) [K,N].  dX or dW may be null to skip it.
int fxp_ref_linear_bwd(const float* dY, const int8_t* Xq, const int8_t* Wq, int32_t eX, int32_t eW, int64_t M,
                       int64_t K, int64_t N, float* dX, float* dW, int8_t* dYq, int32_t* eG, uint64_t seed,
                       uint64_t step, int rounding, int bits) {
    if (!dY || !Xq || !Wq || !dYq || !eG) return -1;
    int rc;
    if ((rc = fxp_ref_scale(dY, static_cast<uint64_t>(M * N), eG))) return rc;
    if ((rc = fxp_ref_map(dY, M, N, *eG, dYq, nullptr, seed, (step << 8) | 2u, rounding, bits))) return rc;
    if (dX && (rc = product_unmap(0, 1, M, K, N, dYq, N, Wq, N, *eG, eW, bits, dX))) return rc;
    if (dW && (rc = product_unmap(1, 0, K, N, M, Xq, K, dYq, N, eX, *eG, bits, dW))) return rc;
    return 0;
}


// ---- convolution (Sec. 3.4, "Linear and convolutional layers": the same integer inner products) ----
// Channels-last tensors: X[N,H,W,C], W[Cout,KH,KW,C], Y and dY [N,Ho,Wo,Cout], zero padding `pad`,
// stride `stride`, Ho = (H + 2 pad - KH) / stride + 1 (same for Wo).  The three functions below are
// the textbook definitions on the int8 mantissas with int32 accumulation.
static bool conv_dims_ok(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Cout, int64_t KH, int64_t KW, int64_t stride,
                         int64_t pad, int64_t* Ho, int64_t* Wo) {
    if (N < 1 || H < 1 || W < 1 || C < 1 || Cout < 1 || KH < 1 || KW < 1 || stride < 1 || pad < 0) return false;
    if (H + 2 * pad < KH || W + 2 * pad < KW) return false;
    *Ho = (H + 2 * pad - KH) / stride + 1;
    *Wo = (W + 2 * pad - KW) / stride + 1;
    return true;
}

int fxp_ref_conv2d_fwd_acc(const int8_t* Xq, int64_t N, int64_t H, int64_t W, int64_t C, const int8_t* Wq, int64_t Cout,
                           int64_t KH, int64_t KW, int64_t stride, int64_t pad, int32_t* acc) {
    int64_t Ho, Wo;
    if (!conv_dims_ok(N, H, W, C, Cout, KH, KW, stride, pad, &Ho, &Wo)) return -2;
    if (!Xq || !Wq || !acc) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo)
                for (int64_t co = 0; co < Cout; ++co) {
                    int32_t sum = 0;
                    for (int64_t kh = 0; kh < KH; ++kh)
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            const int64_t h = ho * stride + kh - pad, w = wo * stride + kw - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;   // zero padding
                            for (int64_t c = 0; c < C; ++c)
                                sum += static_cast<int32_t>(Xq[((n * H + h) * W + w) * C + c]) *
                                       static_cast<int32_t>(Wq[((co * KH + kh) * KW + kw) * C + c]);
                        }
                    acc[((n * Ho + ho) * Wo + wo) * Cout + co] = sum;
                }
    return 0;
}

// dL/dX[n,h,w,c] = sum over (co,kh,kw) with (h + pad - kh) = ho * stride, (w + pad - kw) = wo * stride of
// G[n,ho,wo,co] * W[co,kh,kw,c]  (chain rule through the definition above)
int fxp_ref_conv2d_bwd_input_acc(const int8_t* Gq, const int8_t* Wq, int64_t N, int64_t H, int64_t W, int64_t C, int64_t Cout,
                                 int64_t KH, int64_t KW, int64_t stride, int64_t pad, int32_t* dXacc) {
    int64_t Ho, Wo;
    if (!conv_dims_ok(N, H, W, C, Cout, KH, KW, stride, pad, &Ho, &Wo)) return -2;
    if (!Gq || !Wq || !dXacc) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t h = 0; h < H; ++h)
            for (int64_t w = 0; w < W; ++w)
                for (int64_t c = 0; c < C; ++c) {
                    int32_t sum = 0;
                    for (int64_t kh = 0; kh < KH; ++kh)
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            const int64_t th = h + pad - kh, tw = w + pad - kw;
                            if (th < 0 || tw < 0 || th % stride || tw % stride) continue;
                            const int64_t ho = th / stride, wo = tw / stride;
                            if (ho >= Ho || wo >= Wo) continue;
                            for (int64_t co = 0; co < Cout; ++co)
                                sum += static_cast<int32_t>(Gq[((n * Ho + ho) * Wo + wo) * Cout + co]) *
                                       static_cast<int32_t>(Wq[((co * KH + kh) * KW + kw) * C + c]);
                        }
                    dXacc[((n * H + h) * W + w) * C + c] = sum;
                }
    return 0;
}

// dL/dW[co,kh,kw,c] = sum over (n,ho,wo) of X[n, ho*stride+kh-pad, wo*stride+kw-pad, c] * G[n,ho,wo,co]
// (Acc = int32_t, or int64_t when more than kInt32Terms output pixels are summed)
}  // extern "C"
template <typename Acc>
static int conv2d_bwd_weight_acc(const int8_t* Xq, const int8_t* Gq, int64_t N, int64_t H, int64_t W, int64_t C,
                                 int64_t Cout, int64_t KH, int64_t KW, int64_t stride, int64_t pad, Acc* dWacc) {
    int64_t Ho, Wo;
    if (!conv_dims_ok(N, H, W, C, Cout, KH, KW, stride, pad, &Ho, &Wo)) return -2;
    if (!Xq || !Gq || !dWacc) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t co = 0; co < Cout; ++co)
        for (int64_t kh = 0; kh < KH; ++kh)
            for (int64_t kw = 0; kw < KW; ++kw)
                for (int64_t c = 0; c < C; ++c) {
                    Acc sum = 0;
                    for (int64_t n = 0; n < N; ++n)
                        for (int64_t ho = 0; ho < Ho; ++ho) {
                            const int64_t h = ho * stride + kh - pad;
                            if (h < 0 || h >= H) continue;
                            for (int64_t wo = 0; wo < Wo; ++wo) {
                                const int64_t w = wo * stride + kw - pad;
                                if (w < 0 || w >= W) continue;
                                sum += static_cast<Acc>(Xq[((n * H + h) * W + w) * C + c]) *
                                       static_cast<Acc>(Gq[((n * Ho + ho) * Wo + wo) * Cout + co]);
                            }
                        }
                    dWacc[((co * KH + kh) * KW + kw) * C + c] = sum;
                }
    return 0;
}

extern "C" {
int fxp_ref_conv2d_bwd_weight_acc(const int8_t* Xq, const int8_t* Gq, int64_t N, int64_t H, int64_t W, int64_t C,
                                  int64_t Cout, int64_t KH, int64_t KW, int64_t stride, int64_t pad, int32_t* dWacc) {
    return conv2d_bwd_weight_acc<int32_t>(Xq, Gq, N, H, W, C, Cout, KH, KW, stride, pad, dWacc);
}

int fxp_ref_conv2d_bwd_weight_acc64(const int8_t* Xq, const int8_t* Gq, int64_t N, int64_t H, int64_t W, int64_t C,
                                    int64_t Cout, int64_t KH, int64_t KW, int64_t stride, int64_t pad, int64_t* dWacc) {
    return conv2d_bwd_weight_acc<int64_t>(Xq, Gq, N, H, W, C, Cout, KH, KW, stride, pad, dWacc);
}

// Integer convolution layer, forward: the activation tensor is mapped ONCE as a whole (one scale,
// element index = its channels-last flat index, stream tag 0), the weights likewise (tag 1).
int fxp_ref_conv2d_fwd(const float* X, const float* Wt, int64_t N, int64_t H, int64_t W, int64_t C, int64_t Cout, int64_t KH,
                       int64_t KW, int64_t stride, int64_t pad, float* Y, int8_t* Xq, int8_t* Wq, int32_t* eX, int32_t* eW,
                       uint64_t seed, uint64_t step, int rounding, int bits) {
    int64_t Ho, Wo;
    if (!conv_dims_ok(N, H, W, C, Cout, KH, KW, stride, pad, &Ho, &Wo)) return -2;
    if (!X || !Wt || !Y || !Xq || !Wq || !eX || !eW) return -1;
    int rc;
    if ((rc = fxp_ref_scale(X, static_cast<uint64_t>(N * H * W * C), eX))) return rc;
    if ((rc = fxp_ref_scale(Wt, static_cast<uint64_t>(Cout * KH * KW * C), eW))) return rc;
    if ((rc = fxp_ref_map(X, N * H * W, C, *eX, Xq, nullptr, seed, (step << 8) | 0u, rounding, bits))) return rc;
    if ((rc = fxp_ref_map(Wt, Cout, KH * KW * C, *eW, Wq, nullptr, seed, (step << 8) | 1u, rounding, bits))) return rc;
    const size_t n_out = static_cast<size_t>(N * Ho * Wo * Cout);
    int32_t* acc = new int32_t[n_out + 1];
    rc = fxp_ref_conv2d_fwd_acc(Xq, N, H, W, C, Wq, Cout, KH, KW, stride, pad, acc);
    if (!rc) rc = fxp_ref_unmap(acc, n_out, *eX, bits, *eW, bits, Y);
    delete[] acc;
    return rc;
}

// Backward: the upstream gradient dY[N,Ho,Wo,Cout] is mapped once (tag 2) and used by both gradients.
int fxp_ref_conv2d_bwd(const float* dY, const int8_t* Xq, const int8_t* Wq, int32_t eX, int32_t eW, int64_t N, int64_t H,
                       int64_t W, int64_t C, int64_t Cout, int64_t KH, int64_t KW, int64_t stride, int64_t pad, float* dX,
                       float* dW, int8_t* dYq, int32_t* eG, uint64_t seed, uint64_t step, int rounding, int bits) {
    int64_t Ho, Wo;
    if (!conv_dims_ok(N, H, W, C, Cout, KH, KW, stride, pad, &Ho, &Wo)) return -2;
    if (!dY || !Xq || !Wq || !dYq || !eG) return -1;
    int rc;
    if ((rc = fxp_ref_scale(dY, static_cast<uint64_t>(N * Ho * Wo * Cout), eG))) return rc;
    if ((rc = fxp_ref_map(dY, N * Ho * Wo, Cout, *eG, dYq, nullptr, seed, (step << 8) | 2u, rounding, bits))) return rc;
    if (dX) {
        const size_t n = static_cast<size_t>(N * H * W * C);
        int32_t* acc = new int32_t[n + 1];
        rc = fxp_ref_conv2d_bwd_input_acc(dYq, Wq, N, H, W, C, Cout, KH, KW, stride, pad, acc);
        if (!rc) rc = fxp_ref_unmap(acc, n, *eG, bits, eW, bits, dX);
        delete[] acc;
        if (rc) return rc;
    }
    if (dW) {
        const size_t n = static_cast<size_t>(Cout * KH * KW * C);
        if (N * Ho * Wo <= kInt32Terms) {
            int32_t* acc = new int32_t[n + 1];
            rc = fxp_ref_conv2d_bwd_weight_acc(Xq, dYq, N, H, W, C, Cout, KH, KW, stride, pad, acc);
            if (!rc) rc = fxp_ref_unmap(acc, n, eX, bits, *eG, bits, dW);
            delete[] acc;
        } else {
            int64_t* acc = new int64_t[n + 1];
            rc = fxp_ref_conv2d_bwd_weight_acc64(Xq, dYq, N, H, W, C, Cout, KH, KW, stride, pad, acc);
            if (!rc) rc = fxp_ref_unmap64(acc, n, eX, bits, *eG, bits, dW);
            delete[] acc;
        }
        if (rc) return rc;
    }
    return 0;
}

// ---- batched matrix products (attention: the paper runs Q K^T and A V on the integer mantissas and
// keeps the softmax in floating point; Sec. 5, vision transformer) ----
// `batch` independent products C_b = op(A_b) op(B_b); matrix b of an operand starts b * stride elements
// after matrix 0.  Each product is the plain definition above.
int fxp_ref_gemm_batched(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                         int64_t strideA, const int8_t* B, int64_t ldb, int64_t strideB, int32_t* C, int64_t ldc,
                         int64_t strideC, int64_t batch) {
    if (batch < 0) return -2;
    for (int64_t b = 0; b < batch; ++b) {
        const int rc = fxp_ref_gemm(transA, transB, M, N, K, A + b * strideA, lda, B + b * strideB, ldb, C + b * strideC, ldc);
        if (rc) return rc;
    }
    return 0;
}

// Forward of a batched product layer, Y_b = unmap(map(A)_b * op(map(Bm)_b)).  A[batch,M,K]; Bm[batch,K,N], or
// [batch,N,K] with transB (keys of an attention head: scores = Q K^T).  Each TENSOR gets one scale and is
// mapped once as a whole (row-major element index into the random stream; tags 0 for A, 1 for Bm), exactly
// like the operands of a linear layer.  Aq / Bq come back in the layouts of A / Bm.
int fxp_ref_bmm_fwd(const float* A, const float* Bm, int64_t batch, int64_t M, int64_t K, int64_t N, int transB,
                    float* Y, int8_t* Aq, int8_t* Bq, int32_t* eA, int32_t* eB, uint64_t seed, uint64_t step,
                    int rounding, int bits) {
    if (!A || !Bm || !Y || !Aq || !Bq || !eA || !eB) return -1;
    if (batch < 0 || M < 0 || K < 0 || N < 0) return -2;
    int rc;
    if ((rc = fxp_ref_scale(A, static_cast<uint64_t>(batch * M * K), eA))) return rc;
    if ((rc = fxp_ref_scale(Bm, static_cast<uint64_t>(batch * K * N), eB))) return rc;
    if ((rc = fxp_ref_map(A, batch * M, K, *eA, Aq, nullptr, seed, (step << 8) | 0u, rounding, bits))) return rc;
    const int64_t b_rows = transB ? N : K, b_cols = transB ? K : N;
    if ((rc = fxp_ref_map(Bm, batch * b_rows, b_cols, *eB, Bq, nullptr, seed, (step << 8) | 1u, rounding, bits))) return rc;
    const size_t n = static_cast<size_t>(batch * M * N);
    int32_t* acc = new int32_t[n + 1];
    rc = fxp_ref_gemm_batched(0, transB, M, N, K, Aq, K, M * K, Bq, b_cols, K * N, acc, N, M * N, batch);
    if (!rc) rc = fxp_ref_unmap(acc, n, *eA, bits, *eB, bits, Y);
    delete[] acc;
    return rc;
}

// Backward: G = map(dY[batch,M,N]) once (tag 2); dA_b = unmap(G_b * op(Bq_b)^T) [M,K];
// dBm_b = unmap(Aq_b^T * G_b) [K,N], or its transpose unmap(G_b^T * Aq_b) [N,K] with transB.
int fxp_ref_bmm_bwd(const float* dY, const int8_t* Aq, const int8_t* Bq, int32_t eA, int32_t eB, int64_t batch,
                    int64_t M, int64_t K, int64_t N, int transB, float* dA, float* dBm, int8_t* dYq, int32_t* eG,
                    uint64_t seed, uint64_t step, int rounding, int bits) {
    if (!dY || !Aq || !Bq || !dYq || !eG) return -1;
    if (batch < 0 || M < 0 || K < 0 || N < 0) return -2;
    int rc;
    if ((rc = fxp_ref_scale(dY, static_cast<uint64_t>(batch * M * N), eG))) return rc;
    if ((rc = fxp_ref_map(dY, batch * M, N, *eG, dYq, nullptr, seed, (step << 8) | 2u, rounding, bits))) return rc;
    const int64_t b_cols = transB ? K : N;
    if (dA) {
        const size_t n = static_cast<size_t>(batch * M * K);
        int32_t* acc = new int32_t[n + 1];
        // contraction over N: op(B_b)^T is [N,K], which is Bq_b as stored when transB, else its transpose
        rc = fxp_ref_gemm_batched(0, transB ? 0 : 1, M, K, N, dYq, N, M * N, Bq, b_cols, K * N, acc, K, M * K, batch);
        if (!rc) rc = fxp_ref_unmap(acc, n, *eG, bits, eB, bits, dA);
        delete[] acc;
        if (rc) return rc;
    }
    if (dBm) {
        const size_t n = static_cast<size_t>(batch * K * N);
        int32_t* acc = new int32_t[n + 1];
        if (transB) {   // dBm_b[N,K] = G_b^T[N,M] * Aq_b[M,K]
            rc = fxp_ref_gemm_batched(1, 0, N, K, M, dYq, N, M * N, Aq, K, M * K, acc, K, K * N, batch);
            if (!rc) rc = fxp_ref_unmap(acc, n, *eG, bits, eA, bits, dBm);
        } else {        // dBm_b[K,N] = Aq_b^T[K,M] * G_b[M,N]
            rc = fxp_ref_gemm_batched(1, 0, K, N, M, Aq, K, M * K, dYq, N, M * N, acc, N, K * N, batch);
            if (!rc) rc = fxp_ref_unmap(acc, n, eA, bits, *eG, bits, dBm);
        }
        delete[] acc;
        if (rc) return rc;
    }
    return 0;
}

// ---- int16 weight update (Remark 5, App. A.4: w_hat_{k+1} = w_hat_k + alpha_hat_k * g_hat) ----------------
// One fixed-point "a times y plus x": z = x_hat + SR(a_hat * y_hat), every operand the 16-bit instance of the
// map of Sec. 3.1 (15 magnitude bits: the 24-bit mantissa rounded stochastically with its low 9 bits).
//   x_hat, y_hat : tensors, scales e_x, e_y, units 2^Ex, 2^Ey with E = e_max - 127 - 14
//   a_hat        : the scalar mapped like a one-element tensor (its own exponent is its scale), unit 2^Ea
//   p_i = a_hat * y_hat_i          exact in int32, unit 2^(Ea + Ey)
//   u_i = p_i brought to the unit of x_hat: shifted left when Ea + Ey >= Ex, else shifted right by
//         s = Ex - (Ea + Ey) bits with stochastic rounding of the magnitude: up with probability
//         (dropped bits) / 2^s, decided by word < floor((dropped bits) * 2^32 / 2^s); |u_i| saturates at
//         2^23 - 2^15 so that the sum below stays an exact fp32 mantissa
//   z_i = (x_hat_i + u_i) * 2^Ex   through the inverse mapping of Sec. 3.2
// Random numbers, streams (step << 8) | tag: element i of x and of y round with two disjoint 9-bit fields of
// ONE word (tag 3: bits 31..23 for x, bits 22..14 for y), the update u_i with the full 32-bit word of tag 4,
// the scalar with the top 9 bits of word 0 of tag 5.  rounding = 1 replaces every stochastic rounding by
// round-half-up on the magnitude.
static const uint64_t kTagAxpyXY = 3, kTagAxpyU = 4, kTagAxpyA = 5;
static const int64_t kAxpyUpdateSat = (int64_t{1} << 23) - (int64_t{1} << 15);

static int64_t axpy_update(int32_t p, int32_t s, uint32_t word, int rounding) {
    const bool neg = p < 0;
    const uint64_t m = static_cast<uint64_t>(neg ? -static_cast<int64_t>(p) : static_cast<int64_t>(p));   // < 2^30
    uint64_t u;
    if (s <= 0) {
        u = (-s >= 24) ? (m ? static_cast<uint64_t>(kAxpyUpdateSat) : 0u) : (m << -s);
    } else if (s >= 63) {
        u = 0;                                        // below 2^-33 of a unit: never rounds up
    } else {
        const uint64_t kept = m >> s;
        const uint64_t dropped = m & ((uint64_t{1} << s) - 1u);
        uint64_t up;
        if (rounding == 0) {
            // dropped < 2^30: dropped * 2^32 fits 64 bits
            const uint64_t threshold = (dropped << 32) >> s;       // floor(dropped * 2^32 / 2^s)
            up = (static_cast<uint64_t>(word) < threshold) ? 1u : 0u;
        } else {
            up = (dropped >> (s - 1)) & 1u;                        // half up
        }
        u = kept + up;
    }
    if (u > static_cast<uint64_t>(kAxpyUpdateSat)) u = static_cast<uint64_t>(kAxpyUpdateSat);
    return neg ? -static_cast<int64_t>(u) : static_cast<int64_t>(u);
}

// int16 instance of the map for a flat tensor
int fxp_ref_map16(const float* x, uint64_t n, int32_t e_max, int16_t* q, uint64_t seed, uint64_t stream_id, int rounding) {
    if (n && (!x || !q)) return -1;
    if (rounding < 0 || rounding > 1) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < static_cast<int64_t>(n); ++i)
        q[i] = static_cast<int16_t>(map_one(x[i], e_max, random_word(seed, stream_id, static_cast<uint64_t>(i)), rounding, 16));
    return 0;
}

// z = x + a * y in 16-bit fixed point (see above).  e_out[0..2] receive the scales of x, y and a.
int fxp_ref_axpy16(const float* x, const float* y, float a, uint64_t n, float* z, int32_t* e_out, uint64_t seed,
                   uint64_t step, int rounding) {
    if (n && (!x || !y || !z)) return -1;
    if (rounding < 0 || rounding > 1) return -2;
    int32_t ex, ey, ea;
    int rc;
    if ((rc = fxp_ref_scale(x, n, &ex))) return rc;
    if ((rc = fxp_ref_scale(y, n, &ey))) return rc;
    if ((rc = fxp_ref_scale(&a, 1, &ea))) return rc;
    if (e_out) { e_out[0] = ex; e_out[1] = ey; e_out[2] = ea; }
    const int32_t a_hat = map_one(a, ea, random_word(seed, (step << 8) | kTagAxpyA, 0), rounding, 16);
    const int32_t Ex = lsb_exponent(ex, 16), Ey = lsb_exponent(ey, 16), Ea = lsb_exponent(ea, 16);
    const int32_t s = Ex - (Ea + Ey);
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < static_cast<int64_t>(n); ++k) {
        const uint64_t i = static_cast<uint64_t>(k);
        const uint32_t word_xy = random_word(seed, (step << 8) | kTagAxpyXY, i);
        const int32_t x_hat = map_one(x[i], ex, word_xy, rounding, 16);        // compares bits 31..23
        const int32_t y_hat = map_one(y[i], ey, word_xy << 9, rounding, 16);   // compares bits 22..14
        const int32_t p = a_hat * y_hat;
        const int64_t r = static_cast<int64_t>(x_hat) + axpy_update(p, s, random_word(seed, (step << 8) | kTagAxpyU, i), rounding);
        z[i] = static_cast<float>(std::ldexp(static_cast<double>(r), Ex));
    }
    return 0;
}

// One SGD step with weight decay and momentum (the optimiser of the paper's classification runs, App. A.5:
// momentum 0.9), every line an axpy16:   g1 = g + wd * w;   v = g1 + momentum * v;   w = w + (-lr) * v.
// wd == 0 skips the first line (g1 = g), momentum == 0 the second (v is not touched, the update uses g1).
// tmp: n floats of scratch (may be NULL when wd == 0).  The three lines use steps 3*step, 3*step+1, 3*step+2
// of the random streams.
int fxp_ref_sgd16_step(float* w, const float* g, float* v, uint64_t n, float lr, float momentum, float wd, float* tmp,
                       uint64_t seed, uint64_t step, int rounding) {
    if (n && (!w || !g)) return -1;
    if (momentum != 0.0f && n && !v) return -1;
    if (wd != 0.0f && n && !tmp) return -1;
    int rc;
    const float* g1 = g;
    if (wd != 0.0f) {
        if ((rc = fxp_ref_axpy16(g, w, wd, n, tmp, nullptr, seed, 3 * step, rounding))) return rc;
        g1 = tmp;
    }
    const float* d = g1;
    if (momentum != 0.0f) {
        if ((rc = fxp_ref_axpy16(g1, v, momentum, n, v, nullptr, seed, 3 * step + 1, rounding))) return rc;
        d = v;
    }
    return fxp_ref_axpy16(w, d, -lr, n, w, nullptr, seed, 3 * step + 2, rounding);
}

// The same step for a list of parameter tensors, each with its own scales (one scale per tensor, Sec. 3.1): tensor t
// is updated exactly as fxp_ref_sgd16_step would with the stream step (step << 16) | t, so that no two tensors
// share random numbers.  Arrays of `count` pointers / sizes; v[t] and tmp[t] may be NULL as above.
int fxp_ref_sgd16_step_multi(float* const* w, const float* const* g, float* const* v, float* const* tmp, const uint64_t* n,
                             uint64_t count, float lr, float momentum, float wd, uint64_t seed, uint64_t step, int rounding) {
    if (count > 65536 || step >= (uint64_t{1} << 32)) return -2;
    if (count && (!w || !g || !n)) return -1;
    for (uint64_t t = 0; t < count; ++t) {
        const int rc = fxp_ref_sgd16_step(w[t], g[t], v ? v[t] : nullptr, n[t], lr, momentum, wd, tmp ? tmp[t] : nullptr, seed,
                                          (step << 16) | t, rounding);
        if (rc) return rc;
    }
    return 0;
}

}  // extern "C"
