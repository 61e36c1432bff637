/*
 * fxp.h — C ABI of libfxp: the integer (dynamic fixed-point) layer step of "Is Integer
 * Arithmetic Enough for Deep Learning Training?" (arXiv 2207.08822) - linear, convolution
 * and batched-product layers, forward and backward, and the int16 weight update - as
 * hand-written HIP kernels for gfx950 (MI355X).
 *
 * Conventions that hold for every call
 *  - Every data pointer is a DEVICE pointer unless the argument says "host".
 *    The caller owns every buffer; the library never allocates, frees or keeps
 *    a pointer after the call's work has run.
 *  - All matrices are dense row-major.  X[M,K], W[K,N], Y[M,N], dY[M,N],
 *    dX[M,K], dW[K,N] (the paper's Y = XW, App. A.2).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work; they never synchronise and never read device
 *    memory from the host, so per-tensor scales stay on the device.
 *  - `ws` is device scratch of at least fxp_workspace_bytes(...) bytes, 256-byte
 *    aligned, private to the call until its work has finished on `stream`.
 *  - Return value: FXP_OK (0) or a negative fxp_status; nothing is enqueued when
 *    an argument error is returned.  Launch failures reported by the runtime map
 *    to FXP_ERR_LAUNCH.  No exception crosses this boundary.
 *  - A mapped tensor is int8 values q plus ONE int32 scale e_max (the biased
 *    fp32 exponent field of its largest magnitude, Sec. 3.1); q stands for the
 *    real number q * 2^(e_max - 127 - (bits - 2)), i.e. q * 2^(e_max - 133) for
 *    the paper's int8 (bits = 8: sign + 7 magnitude bits).
 *  - Inputs must be finite.  Non-finite input is not an error (it cannot be seen
 *    without a synchronisation): the scale then reads 255, +-Inf maps to the
 *    largest magnitude and NaN to 0.
 */
#ifndef FXP_H_
#define FXP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fxp_status {
    FXP_OK = 0,
    FXP_ERR_NULL = -1,      /* a required pointer is NULL */
    FXP_ERR_DIMS = -2,      /* negative size, leading dimension too small, or size beyond the supported range */
    FXP_ERR_ALIGN = -3,     /* a pointer misses the alignment stated for it */
    FXP_ERR_WORKSPACE = -4, /* ws is NULL or smaller than fxp_workspace_bytes says */
    FXP_ERR_ROUNDING = -5,  /* unknown rounding mode */
    FXP_ERR_BITS = -6,      /* bits outside [2, 8] */
    FXP_ERR_LAUNCH = -7,    /* the HIP runtime refused a launch */
    FXP_ERR_OVERFLOW = -8   /* contraction longer than an int32 sum is sure to hold (> 133144 terms) where the call has no
                               64-bit path for it: int32 output, a batched product, or no room in ws for the slices */
} fxp_status;

/* Rounding of the 24-bit shifted mantissa to bits-1 magnitude bits. */
enum {
    FXP_ROUND_STOCHASTIC = 0, /* App. A.1: up with probability (dropped bits) / 2^(number dropped) */
    FXP_ROUND_NEAREST = 1     /* half up on the magnitude; for comparison runs only */
};

/* Operation selector of fxp_workspace_bytes. */
enum { FXP_OP_SCALE = 0, FXP_OP_GEMM = 1, FXP_OP_LINEAR_FWD = 2, FXP_OP_LINEAR_BWD = 3, FXP_OP_BMM_FWD = 4, FXP_OP_BMM_BWD = 5 };

/* Random-stream tags of the layer calls: stream_id = (step << 8) | tag. */
enum { FXP_TAG_X = 0, FXP_TAG_W = 1, FXP_TAG_DY = 2 };

/* Host string for a status code (static storage). */
const char* fxp_strerror(int status);

/* Library version, major * 100 + minor. */
int fxp_version(void);

/* Scratch bytes an operation needs.  FXP_OP_SCALE: M = number of elements.
 * FXP_OP_GEMM: worst case over the operand forms of fxp_gemm / fxp_gemm_unmap.
 * FXP_OP_GEMM includes the int32 slices a long, narrow product is split into along K.
 * FXP_OP_BMM_FWD / _BWD: scale scratch only, whatever the shapes.
 * FXP_OP_LINEAR_FWD / _BWD: layer shapes M, N, K as above.  Returns 0 on bad
 * arguments. */
size_t fxp_workspace_bytes(int op, int64_t M, int64_t N, int64_t K);

/* Scale of a tensor (Sec. 3.1: e_max = max(e_1 .. e_n)).
 * x: n fp32 values, 4-byte aligned, any n >= 0.  e_max: one int32, receives the
 * largest biased exponent field, counting zeros and sub-normals as 1, so the
 * result lies in [1, 255] (n = 0 gives 1). */
int fxp_scale(const float* x, size_t n, int32_t* e_max, void* ws, size_t ws_bytes, void* stream);

/* Linear fixed-point mapping (Sec. 3.1; stochastic rounding of App. A.1, Fig. 4).
 * x: [rows, cols] fp32.  e_max: the tensor's scale as fxp_scale wrote it (a
 * larger value is allowed, e.g. a scale shared between shards; elements whose
 * exponent exceeds it saturate).  q: [rows, cols] int8 or NULL.  qT: [cols,
 * rows] int8 or NULL, the same values transposed (one rounding decision per
 * element, shared by both copies).  At least one of q, qT is required.
 * Per element: 24-bit mantissa (hidden bit restored) shifted right by
 * e_max - e, cut after bits-1 magnitude bits, rounded up iff r < dropped bits,
 * saturated to 2^(bits-1) - 1, sign attached.  r is the top (25 - bits) bits
 * of word (i mod 4) of Philox-4x32-10 with key = seed and counter =
 * (i / 4, stream_id), i = row * cols + col: the result does not depend on the
 * launch geometry or on which copies are requested.
 * Fast path: x, q, qT 16-byte aligned and cols a multiple of 4; anything else
 * takes a slower element-wise kernel with identical results. */
int fxp_map(const float* x, int64_t rows, int64_t cols, const int32_t* e_max, int8_t* q, int8_t* qT, uint64_t seed,
            uint64_t stream_id, int rounding, int bits, void* stream);

/* fxp_scale followed by fxp_map with the final reduction folded into the map
 * kernel: writes *e_max and q / qT exactly as the two calls would. */
int fxp_scale_map(const float* x, int64_t rows, int64_t cols, int32_t* e_max, int8_t* q, int8_t* qT, uint64_t seed,
                  uint64_t stream_id, int rounding, int bits, void* ws, size_t ws_bytes, void* stream);

/* Two tensors per launch: what fxp_map / fxp_scale_map do for one tensor, done for two with one map launch
 * (and one reduction launch) instead of two each - the layer calls use this for the activation and the
 * weight of a forward pass, where the second tensor is often too small to fill the chip by itself.  Results
 * are identical to two separate calls.  One launch needs both tensors on the fast path of fxp_map and of the
 * same tile width (cols <= 64 or cols % 128 in 1..64 selects the narrow tile); otherwise two launches are made. */
typedef struct fxp_map_desc {
    const float* x;      /* [rows, cols] fp32, device */
    int64_t rows, cols;
    int32_t* e_max;      /* device: read by fxp_map2, written by fxp_scale_map2 */
    int8_t* q;           /* [rows, cols] or NULL */
    int8_t* qT;          /* [cols, rows] or NULL */
    uint64_t stream_id;
} fxp_map_desc;
int fxp_map2(const fxp_map_desc* a, const fxp_map_desc* b, uint64_t seed, int rounding, int bits, void* stream);
/* ws: device, >= 2 * fxp_workspace_bytes(FXP_OP_SCALE, ...) bytes */
int fxp_scale_map2(const fxp_map_desc* a, const fxp_map_desc* b, uint64_t seed, int rounding, int bits, void* ws,
                   size_t ws_bytes, void* stream);

/* Number of uint32 words of an abs-max area (see fxp_gemm_unmap_absmax). */
#define FXP_ABSMAX_WORDS 256

/* fxp_map with the scale taken from the largest magnitude of the tensor, given as an abs-max area: device
 * array of FXP_ABSMAX_WORDS uint32 whose maximum is the IEEE bit pattern of max |x_i| (what
 * fxp_gemm_unmap_absmax leaves behind for its output).  The scale of Sec. 3.1 is the exponent field of that
 * maximum, at least 1.  It is written to *e_max (required) and used for the mapping in the same launch, so a
 * tensor produced by a product of this library is mapped without a reduction pass of its own.  An area below
 * the tensor's true maximum gives a scale below the tensor (elements above it saturate), as a too small e_max
 * does for fxp_map. */
int fxp_map_absmax(const float* x, int64_t rows, int64_t cols, const uint32_t* absmax, int32_t* e_max, int8_t* q, int8_t* qT,
                   uint64_t seed, uint64_t stream_id, int rounding, int bits, void* stream);

/* Integer GEMM (Sec. 3.3, Fig. 2: int8 x int8 products, int32 accumulation).
 * C[M,N] = op(A)[M,K] * op(B)[K,N], C overwritten.
 * transA = 0: A stored [M,K], lda >= K.  transA = 1: A stored [K,M], lda >= M.
 * transB = 0: B stored [K,N], ldb >= N.  transB = 1: B stored [N,K], ldb >= K.
 * Native form is (transA, transB) = (0, 1), both operands contiguous along the
 * contraction; other forms first transpose the operand into ws.  K <= 133144 (127^2 * K < 2^31: the int32
 * sums cannot wrap).
 * Fast loads need A, B 16-byte aligned and lda, ldb, K multiples of 16; other
 * shapes take a slower loader with identical results.  C 4-byte aligned. */
int fxp_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, const int8_t* B,
             int64_t ldb, int32_t* C, int64_t ldc, void* ws, size_t ws_bytes, void* stream);

/* Non-linear inverse mapping (Sec. 3.2, Fig. 1b) of an integer tensor with the
 * shared exponent of Sec. 3.3 (sum of the operand exponents):
 * out = fp32 nearest (ties to even, gradual underflow, overflow to Inf) to
 * acc * 2^E, E = (eA - 127 - (bitsA-2)) + (eB - 127 - (bitsB-2)); eB = NULL
 * drops the second term.  acc and out may be the same buffer. */
int fxp_unmap(const int32_t* acc, size_t n, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB, float* out,
              void* stream);

/* Inverse mapping of a mapped int8 tensor itself: out = q * 2^(eA - 127 - (bitsA-2)). */
int fxp_unmap_i8(const int8_t* q, size_t n, const int32_t* eA, int bitsA, float* out, void* stream);

/* fxp_gemm with the inverse mapping fused into its epilogue: C is fp32 and
 * receives what fxp_unmap would make of the int32 result.
 * K may exceed 133144 here: the contraction then runs as slices of at most 133120 terms, each summed exactly
 * in int32 into ws, and the slices are added in 64 bits before the one rounding of the inverse mapping - C is
 * the exact integer sum times 2^E, rounded once, at any K < 2^31.  That needs the ws of
 * fxp_workspace_bytes(FXP_OP_GEMM, M, N, K); with less, FXP_ERR_OVERFLOW. */
int fxp_gemm_unmap(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                   const int8_t* B, int64_t ldb, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB, float* C,
                   int64_t ldc, void* ws, size_t ws_bytes, void* stream);

/* fxp_gemm_unmap that also leaves the largest output magnitude behind, so that the next layer can map C without
 * a reduction pass over it (Sec. 3.1's scale is the exponent field of that magnitude).  out_absmax (required):
 * device array of FXP_ABSMAX_WORDS uint32, 4-byte aligned; the call raises its words by atomic maxima so that
 * their maximum is at least the IEEE bit pattern of max |C_ij| (several words, so that the workgroups do not
 * all hit one address).  The caller zeroes the area before the first product that contributes to a tensor
 * (several products may fill parts of one tensor).  Consumed by fxp_map_absmax.  Everything else as
 * fxp_gemm_unmap. */
int fxp_gemm_unmap_absmax(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                          const int8_t* B, int64_t ldb, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                          float* C, int64_t ldc, uint32_t* out_absmax, void* ws, size_t ws_bytes, void* stream);

/* Mapped operands a forward call leaves for the backward call (host struct of
 * device pointers, all caller-allocated, 16-byte aligned). */
typedef struct fxp_saved {
    int8_t* Xq;   /* [M,K] */
    int8_t* XqT;  /* [K,M] */
    int8_t* Wq;   /* [K,N] */
    int8_t* WqT;  /* [N,K] */
    int32_t* eX;  /* 1 */
    int32_t* eW;  /* 1 */
} fxp_saved;

/* Forward of one integer linear layer (App. A.2: Y_hat = X_hat W_hat):
 * scale + map X (stream tag FXP_TAG_X), scale + map W (FXP_TAG_W), int8 GEMM,
 * inverse mapping -> Y[M,N] fp32.  Fills every member of *saved. */
int fxp_linear_fwd(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y, const fxp_saved* saved,
                   uint64_t seed, uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream);

/* fxp_linear_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments without ws, same results bit
 * for bit; the call allocates and frees nothing.  Its scratch (block maxima of the two scale reductions, int32
 * slices of a product that is split along its contraction) is a device array of FXP_STATIC_SCRATCH_BYTES bytes
 * inside the library, one copy per GPU, held until the process ends.  A layer that needs more -
 * fxp_workspace_bytes(FXP_OP_LINEAR_FWD, M, N, K) > FXP_STATIC_SCRATCH_BYTES, which only long contractions into
 * small outputs reach - returns FXP_ERR_WORKSPACE and enqueues nothing.  All calls on one GPU share that GPU's
 * array: two calls whose work overlaps in time on one GPU (different streams, or different threads) race;
 * calls on one stream are ordered and safe.  The array's previous contents never matter (every word read was
 * written by the same call).  The first call on a device looks the array's address up (no allocation), so make
 * one call per device before a capture begins. */
#define FXP_STATIC_SCRATCH_BYTES (32u << 20)
size_t fxp_static_scratch_bytes(void);
int fxp_linear_fwd_static(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y, const fxp_saved* saved,
                          uint64_t seed, uint64_t step, int rounding, int bits, void* stream);

/* Backward of the same layer (App. A.2: dL/dW = X_hat^T G_hat; chain rule for
 * dL/dX = G_hat W_hat^T): scale + map dY ONCE (FXP_TAG_DY; both GEMMs use the
 * same rounded gradient), then dX[M,K] and dW[K,N] as fp32.  dX or dW may be
 * NULL to skip it.  dYq [M,N], dYqT [N,M] and e_dY (1 int32) are caller-
 * allocated outputs/scratch.  Uses saved->XqT, saved->Wq, saved->eX, saved->eW.
 * M, K, N are not limited by the int32 accumulator: a contraction of more than 133144 terms (the weight
 * gradient of a layer applied to more rows than that) runs as slices, see fxp_gemm_unmap. */
int fxp_linear_bwd(const float* dY, const fxp_saved* saved, int64_t M, int64_t K, int64_t N, float* dX, float* dW,
                   int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step, int rounding, int bits,
                   void* ws, size_t ws_bytes, void* stream);

/* The same two calls for a training loop, where a tensor's scale seldom moves from one step to the next (Sec. 3.1:
 * the scale is the largest exponent of the tensor).  saved->eX, saved->eW and e_dY are read on entry as GUESSES of
 * the scales (what the previous step's call left there; any other content is harmless).  Each large tensor is then
 * read ONCE: a single pass maps it with the guess and finds its true largest magnitude, and a second, short launch
 * verifies - if the guess was the scale, the mapped tensor is already what fxp_linear_fwd / _bwd would have
 * written; if not (the maximum crossed a power of two, first call, garbage in the word), that launch maps the
 * tensor again with the true scale.  Results are bit for bit those of fxp_linear_fwd / fxp_linear_bwd in every
 * case; a hit saves the reduction's pass over the tensor (4 of 10 bytes per element), a miss costs one map pass
 * more.  Tensors below 2^22 elements and tensors off the fast path of fxp_map take the two-pass path as before. */
int fxp_linear_fwd_guess(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y, const fxp_saved* saved,
                         uint64_t seed, uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream);
int fxp_linear_bwd_guess(const float* dY, const fxp_saved* saved, int64_t M, int64_t K, int64_t N, float* dX, float* dW,
                         int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step, int rounding, int bits,
                         void* ws, size_t ws_bytes, void* stream);

/* Batched integer GEMM for the attention products (the paper runs Q K^T and A V as int8 matmuls with the
 * softmax in floating point, Sec. 5 / ViT): `batch` (<= 65535) independent products in the native form
 * C_b[M,N] = A_b[M,K] * B_b[N,K]^T, matrix b of an operand starting b * stride elements after matrix 0.
 * One scale per TENSOR (all matrices of A share eA, all of B share eB), as everywhere in the method.
 * Fast loads need 16-byte aligned bases, and lda, ldb, strideA, strideB, K multiples of 16. */
int fxp_gemm_batched(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, int64_t strideA, const int8_t* B,
                     int64_t ldb, int64_t strideB, int32_t* C, int64_t ldc, int64_t strideC, int64_t batch, void* stream);

int fxp_gemm_unmap_batched(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, int64_t strideA, const int8_t* B,
                           int64_t ldb, int64_t strideB, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB, float* C,
                           int64_t ldc, int64_t strideC, int64_t batch, void* stream);

/* Mapped operands of a batched product layer (host struct of device pointers, caller-allocated, 16-byte
 * aligned).  Each tensor is mapped ONCE as a whole, as a matrix of (batch * rows) x cols, in both orientations:
 *   Aq [batch*M, K]      AqT [K, batch*M]
 *   Bq  as Bm is laid out: [batch*K, N], or [batch*N, K] with transB;   BqT its transpose
 * so that every one of the three products per matrix reads K-contiguous operands through a leading dimension
 * and a batch stride alone (matrix b of a transposed copy is a block of columns). */
typedef struct fxp_bmm_saved {
    int8_t* Aq;
    int8_t* AqT;
    int8_t* Bq;
    int8_t* BqT;
    int32_t* eA;  /* 1 */
    int32_t* eB;  /* 1 */
} fxp_bmm_saved;

/* Forward of a batched product layer, the attention matmuls of the vision transformer (Sec. 5: Q K^T and A V
 * run on the integer mantissas, the softmax stays in floating point): Y_b = unmap(map(A)_b * op(map(Bm)_b)),
 * b < batch <= 65535.  A[batch,M,K] fp32; Bm[batch,K,N], or [batch,N,K] with transB != 0 (keys: scores =
 * Q K^T); Y[batch,M,N] fp32.  One scale per tensor; random streams FXP_TAG_X for A, FXP_TAG_W for Bm, element
 * index = row-major index in the whole tensor.  Fills every member of *saved.  Full speed needs M, K, N
 * multiples of 16 (pad the sequence length); other sizes take the slower general loads, same results.
 * ws: fxp_workspace_bytes(FXP_OP_BMM_FWD, ...) bytes, 256-byte aligned. */
int fxp_bmm_fwd(const float* A, const float* Bm, int64_t batch, int64_t M, int64_t K, int64_t N, int transB, float* Y,
                const fxp_bmm_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits, void* ws,
                size_t ws_bytes, void* stream);

/* Backward: dY[batch,M,N] is mapped once (FXP_TAG_DY; dYq [batch*M,N], dYqT [N,batch*M], e_dY returned);
 * dA_b = unmap(G_b * op(Bq_b)^T) [batch,M,K]; dBm_b = unmap(Aq_b^T * G_b), in the layout of Bm.  dA or dBm may
 * be NULL to skip it. */
int fxp_bmm_bwd(const float* dY, const fxp_bmm_saved* saved, int64_t batch, int64_t M, int64_t K, int64_t N,
                int transB, float* dA, float* dBm, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed,
                uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream);

/* fxp_bmm_fwd / fxp_bmm_bwd with the scales saved->eA, saved->eB and e_dY hold on entry taken as guesses: see
 * fxp_linear_fwd_guess.  Same results bit for bit. */
int fxp_bmm_fwd_guess(const float* A, const float* Bm, int64_t batch, int64_t M, int64_t K, int64_t N, int transB, float* Y,
                      const fxp_bmm_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits, void* ws,
                      size_t ws_bytes, void* stream);
int fxp_bmm_bwd_guess(const float* dY, const fxp_bmm_saved* saved, int64_t batch, int64_t M, int64_t K, int64_t N,
                      int transB, float* dA, float* dBm, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed,
                      uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream);

/* ---- int16 weight update (Remark 5, App. A.4: w_hat_{k+1} = w_hat_k + alpha_hat_k * g_hat, every term in fixed
 * point with stochastic rounding; the paper's runs use "int16 SGD", Sec. 5) ----
 * fxp_axpy16: z = x_hat + SR(a_hat * y_hat) over n elements.  x_hat, y_hat, a_hat are the 16-bit instance of
 * the mapping (15 magnitude bits, scale = largest exponent of the tensor; the scalar's scale is its own
 * exponent); the int32 product is brought to the unit of x_hat by a shift, with stochastic rounding of the
 * dropped bits, saturating at 2^23 - 2^15 units; the integer sum goes through the inverse mapping.  The paper
 * does not spell this formula out: alignment and place of the rounding are this library's reading.
 * x, y, z: device, fp32; z may be x or y (in place).  e_out: device int32[3] receiving the scales of x, y, a,
 * or NULL.  Random streams (step << 8) | 3..6.  ws: device, >= 2 * fxp_workspace_bytes(FXP_OP_SCALE) bytes. */
int fxp_axpy16(const float* x, const float* y, float a, size_t n, float* z, int32_t* e_out, uint64_t seed,
               uint64_t step, int rounding, void* ws, size_t ws_bytes, void* stream);

/* One SGD step with weight decay and momentum (the optimiser of the paper's classification runs), every line
 * an fxp_axpy16 with stream steps 3*step, 3*step+1, 3*step+2:
 *   g1 = g + weight_decay * w      (skipped when weight_decay == 0; needs tmp[n])
 *   v  = g1 + momentum * v         (skipped when momentum == 0; v may then be NULL)
 *   w  = w + (-lr) * v             (g1 in place of v without momentum)
 * w, v are updated in place; g is read only.  The scales of the intermediates come out of the producing
 * kernel, so the step reads w, g, v once for their scales and once per line.
 * ws: device, fxp_sgd16_workspace_bytes() bytes. */
size_t fxp_sgd16_workspace_bytes(void);
int fxp_sgd16_step(float* w, const float* g, float* v, size_t n, float lr, float momentum, float weight_decay, float* tmp,
                   uint64_t seed, uint64_t step, int rounding, void* ws, size_t ws_bytes, void* stream);

/* The same step for a whole list of parameter tensors, each with its own scales (the method keeps one scale per
 * tensor), in four launches per 64 tensors instead of six per tensor: what a model with dozens of parameter
 * tensors needs, since a dependent launch costs several microseconds.  Tensor t is updated exactly as
 * fxp_sgd16_step would update it with the stream step (step << 16) | t (so no two tensors share random numbers);
 * count <= 65536, step < 2^32.  `tensors` is a HOST array of device pointers (v may be NULL without momentum,
 * tmp without weight decay; n = 0 entries are skipped); it is only read during the call.
 * ws: device, fxp_sgd16_multi_workspace_bytes(tensors, count) bytes. */
typedef struct fxp_sgd_tensor {
    float* w;
    const float* g;
    float* v;
    float* tmp;
    size_t n;
} fxp_sgd_tensor;
size_t fxp_sgd16_multi_workspace_bytes(const fxp_sgd_tensor* tensors, size_t count);
int fxp_sgd16_step_multi(const fxp_sgd_tensor* tensors, size_t count, float lr, float momentum, float weight_decay,
                         uint64_t seed, uint64_t step, int rounding, void* ws, size_t ws_bytes, void* stream);

/* ---- convolution layer (Sec. 3.4: "Linear and convolutional layers" share the integer inner product) ----
 * Channels-last tensors: X[N,H,W,C], W[Cout,KH,KW,C], Y and dY [N,Ho,Wo,Cout] with
 * Ho = (H + 2 pad - KH) / stride + 1 (same for Wo), zero padding.  Host struct. */
typedef struct fxp_conv2d_shape {
    int64_t N, H, W, C, Cout, KH, KW, stride, pad;
} fxp_conv2d_shape;

/* What a forward call leaves for the backward call (host struct of device pointers, caller-allocated,
 * 16-byte aligned): the int8 activation itself, the int8 weights in both orientations, the scales. */
typedef struct fxp_conv_saved {
    int8_t* Xq;   /* [N,H,W,C] */
    int8_t* Wq;   /* [Cout, KH*KW*C] */
    int8_t* WqT;  /* [KH*KW*C, Cout] */
    int8_t* WqF;  /* [C, KH*KW*Cout]: kernel flipped in both spatial axes; scratch of the backward call, which
                     fills it from Wq when it computes the input gradient of a stride-1 convolution */
    int32_t* eX;  /* 1 */
    int32_t* eW;  /* 1 */
} fxp_conv_saved;

/* Scratch bytes of fxp_conv2d_fwd (backward = 0) or fxp_conv2d_bwd (backward = 1); 0 on a bad shape. */
size_t fxp_conv2d_workspace_bytes(const fxp_conv2d_shape* shape, int backward);

/* Forward: the activation tensor is mapped once as a whole (element index = its channels-last flat index,
 * FXP_TAG_X), the weights likewise (FXP_TAG_W); the int8 patches are multiplied on the matrix cores - read
 * straight from the int8 activation by the GEMM loader when C is a multiple of 64, gathered into scratch
 * first otherwise - and Y receives the inverse-mapped fp32 result.  Contractions KH*KW*C and KH*KW*Cout <= 133144. */
int fxp_conv2d_fwd(const float* X, const float* W, const fxp_conv2d_shape* shape, float* Y, const fxp_conv_saved* saved,
                   uint64_t seed, uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream);

/* Backward: dY is mapped once (FXP_TAG_DY); dW[Cout,KH,KW,C] sums over all N*Ho*Wo output pixels (any number: beyond
 * 133144 the sum runs as int32 slices added in 64 bits, like the long contractions of fxp_gemm_unmap),
 * dX[N,H,W,C] sums, per input pixel, the patch entries that read it (exact int32, then one inverse mapping).
 * dX or dW may be NULL.  dYq [N*Ho*Wo, Cout], dYqT [Cout, N*Ho*Wo] and e_dY are caller-allocated. */
int fxp_conv2d_bwd(const float* dY, const fxp_conv_saved* saved, const fxp_conv2d_shape* shape, float* dX, float* dW,
                   int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step, int rounding, int bits,
                   void* ws, size_t ws_bytes, void* stream);

/* ---- measurement helper (not a step of the method) ----
 * Core clock while other work runs: enqueues one wave on `stream` (use a stream of its own, next to the kernels
 * under test) that stays alive for `microseconds` (1 .. 1000000) of the constant 100 MHz counter and then writes
 * out[0] = ticks of that counter, out[1] = core clock cycles in the same interval (device, 2 x uint64, 8-byte
 * aligned): core clock in MHz = 100 * out[1] / out[0].  The compute-bound products of Sec. 3.3 run the chip
 * into its power limit, so their rate is reported next to the clock they ran at. */
int fxp_clock_probe(uint64_t* out, uint32_t microseconds, void* stream);

/* Time stamps inside the linear-layer calls.  After fxp_timeline_begin(capacity) (host call; creates `capacity`
 * HIP events, 1 .. 2^20) every fxp_linear_fwd / fxp_linear_bwd records one event on its stream at its entry
 * (FXP_TL_ENTRY) and one after each of its launches, tagged with what the launch was, until the events are used
 * up.  fxp_timeline_end waits for the last recorded event and returns, for every pair of consecutive events, the
 * elapsed microseconds and the tag of the later one (so an interval is the in-stream duration of that launch
 * behind the launch that really precedes it in the step; an FXP_TL_ENTRY interval is the idle time between two
 * calls); *count receives the number of intervals written (at most `capacity`).  Then the events are destroyed.
 * One timeline per process; not to be begun or ended while layer calls are running in other threads. */
enum { FXP_TL_ENTRY = 0, FXP_TL_SCALE = 1, FXP_TL_MAP = 2, FXP_TL_GEMM_FWD = 3, FXP_TL_GEMM_DW = 4, FXP_TL_GEMM_DX = 5,
       FXP_TL_REDUCE = 6 };
int fxp_timeline_begin(int capacity);
int fxp_timeline_end(float* microseconds, int* tags, int capacity, int* count);

#ifdef __cplusplus
}
#endif
#endif /* FXP_H_ */
