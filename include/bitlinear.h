/*
 * bitlinear.h - C-ABI of the BitLinear W1.58A8 hot path for AMD MI355X (gfx950).
 *
 * The operation is the BitLinear layer of BitNet b1.58 (technical report,
 * Section 2 "Architecture": absmean ternary weights, per-token absmax int8
 * activations; Section 5.1 "GPU Inference": four ternary values stored per
 * 8-bit integer, unpacked just before the integer matrix product).
 *
 * The report gives these steps in words only.  The arithmetic below is the
 * reading this library fixes; every fp32 step is ONE IEEE-754 binary32
 * round-to-nearest-even operation, in the order written, with no fused
 * multiply-add contraction.
 *
 *   weight scale   beta = fp32( (sum_{n,k} |W[n][k]|) / (N*K) )      (sum and
 *                  division carried in fp64, one final rounding to fp32)
 *   ternarize      d = beta + 1e-5f ; t = rint(W[n][k] / d) (ties to even);
 *                  Wt[n][k] = clamp(t, -1, +1)  in {-1, 0, +1}
 *   code           c = Wt + 1  in {0, 1, 2}        (3 is never produced)
 *   activation     x~ = fp32(bf16 X[m][k]) ; gamma = max_k |x~| ;
 *   quantizer      g = max(gamma, 1e-5f) ; inv = 127.0f / g ;
 *                  q[m][k] = clamp(rint(x~ * inv), -127, 127)  (ties to even);
 *                  scale[m] = g / 127.0f ; rowsum[m] = sum_k q[m][k]  (int32)
 *   contraction    acc[m][n] = sum_k q[m][k] * Wt[n][k]      (exact, int32)
 *   rescale        y[m][n] = (float)acc[m][n] * (beta * scale[m])
 *
 * PACKED LAYOUTS.  2 bits per weight.  Rows are padded: Kp = bl_padded_k(K) (K rounded up to
 * a multiple of 64) weights per row and Np = N rounded up to a multiple of 4 rows; every field
 * outside the N x K matrix holds code 1 (weight 0).  A packed matrix is Np*Kp/4 bytes
 * (= N*K/4 when K % 64 == 0 and N % 4 == 0).
 *   BL_LAYOUT_ROWMAJOR (0): byte index b = n*(Kp/4) + k/4 ; weight k occupies
 *     bits [2*(k%4), 2*(k%4)+1] of byte b (lowest bits = lowest k).
 *   BL_LAYOUT_K16 (1): same byte count and the same 4-byte word per group of
 *     16 consecutive k of a row, but inside the word the two index digits are
 *     swapped: with i = k % 16, weight k occupies bits [2*(i/4), 2*(i/4)+1] of
 *     byte n*(Kp/4) + (k/16)*4 + i%4.  (So `(word >> 2s) & 0x03030303` yields the
 *     codes of k = 4s..4s+3 as four bytes in natural order: the kernels' native
 *     form.  Layout 0 is supported by permuting the activation bytes instead.)
 *   BL_LAYOUT_TRIT5 (2): five weights per byte, 1.6 bits per weight (the density behind the
 *     memory footprint of Table 1; the 2-bit forms above are the ones Section 5.1 describes).
 *     Rows of Kq = K rounded up to a multiple of 80 weights (Kq/5 bytes, a whole number of
 *     16-byte loads), Np rows, code 1 outside the matrix: Np*Kq/5 bytes.  Inside a row, the 4-byte
 *     word g covers k = 20g .. 20g+19; its byte j holds the codes c_i of k = 20g + 4i + j,
 *     i = 0..4, as b = ceil(v * 256 / 243) with v = sum_i c_i * 3^(4-i) (so that c_0 = (3b) >> 8,
 *     and the same step on the low byte of 3b yields c_1, and so on: no table, no division).
 *     Accepted by bl_pack_ternary, bl_unpack_ternary, bl_packed_bytes and bl_stack_build (the
 *     bandwidth-bound M = 1 decode, where bytes are time); BL_ERR_LAYOUT elsewhere.
 *   BL_LAYOUT_KMAJOR (3): the transposed matrix, one row per input feature k (K rows, no padding
 *     of K), each row the 2-bit codes of n = 0 .. Nq-1, Nq = N rounded up to a multiple of 64, packed
 *     like layout 0 along n (byte index k*(Nq/4) + n/4, bits [2*(n%4), 2*(n%4)+1]), code 1 behind
 *     column N: K*Nq/4 bytes.  For activations that are mostly zero (Section 2 takes squared ReLU
 *     for the sparsity it gives the input of the down projection): the rows of zero activations
 *     are never read.  N <= 3072.  Accepted by bl_pack_ternary, bl_unpack_ternary,
 *     bl_packed_bytes and bl_stack_build; BL_ERR_LAYOUT elsewhere.
 * QUANTISED ACTIVATIONS are int8 [M][Kp]: leading dimension Kp, zeros in columns K..Kp-1 (what
 * bl_quant_act_int8 writes), so that a padded weight meets a zero.  Outputs are [M][N].
 *
 * CONVENTIONS.  Every pointer is a DEVICE pointer owned by the caller unless a
 * comment says "host".  The library allocates and frees nothing; all work is
 * enqueued on the caller's stream `s` (a hipStream_t passed as void*; NULL is
 * the null stream) and no call synchronises.  Argument errors are found on the
 * host before any HIP call and reported as a status code (no exceptions, no
 * global error state; the only process-wide state is the test hook below).  Preconditions on
 * every matrix: 1 <= N, K <= 2^24; `packed` and `q` 16-byte aligned; otherwise
 * BL_ERR_SHAPE / BL_ERR_ALIGN.  Entry points that read bf16 or fp32 activations inside a
 * product kernel (fused producers, epilogues, bl_stack_* with X) need K % 64 == 0 and say so;
 * a ragged K goes through bl_quant_act_int8 and the int8 inputs of the products.
 * Non-finite activations or weights: undefined.
 * There is no bias argument (the report removes all biases, Section 2).
 */
#ifndef BITLINEAR_H
#define BITLINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BL_OK            = 0,
    BL_ERR_NULL      = 1,  /* a required pointer is NULL                        */
    BL_ERR_SHAPE     = 2,  /* M/N/K out of range or not a permitted multiple    */
    BL_ERR_LAYOUT    = 3,  /* unknown layout id / layout not valid for shape    */
    BL_ERR_ALIGN     = 4,  /* pointer not aligned as required                   */
    BL_ERR_VALUE     = 5,  /* unknown in_kind / op id                           */
    BL_ERR_HIP       = 6,  /* a HIP runtime call or kernel launch failed        */
    BL_ERR_WORKSPACE = 7   /* workspace required but NULL                       */
} bl_status;

typedef void* bl_stream;   /* hipStream_t */

enum { BL_LAYOUT_ROWMAJOR = 0, BL_LAYOUT_K16 = 1, BL_LAYOUT_TRIT5 = 2, BL_LAYOUT_KMAJOR = 3 };
enum { BL_IN_FP32_LATENT = 0, BL_IN_INT8_TERNARY = 1 };
enum { BL_OP_PACK = 0, BL_OP_QUANT = 1, BL_OP_GEMV = 2, BL_OP_GEMM = 3 };

/* Library version (major*10000 + minor*100 + patch) and a static string
 * naming a status code.  Host-only, no GPU needed. */
int         bl_version(void);
const char* bl_status_str(int status);

/* Bytes of a packed N x K matrix (Np*Kp/4 for every layout, see PACKED LAYOUTS); 0 if the
 * shape or layout is not permitted.  Host-only.  (Section 5.1: 4 values per byte.) */
size_t bl_packed_bytes(int64_t N, int64_t K, int layout);

/* Kp: K rounded up to a multiple of 64, the row length of packed weights and the leading
 * dimension of quantised activations; 0 if K is out of range.  Host-only. */
int64_t bl_padded_k(int64_t K);

/* Bytes of device scratch the given op needs for the given shape (may be 0).
 * The workspace is caller-allocated, 256-byte aligned, and may be reused by
 * later calls on the same stream.  Host-only. */
size_t bl_workspace_bytes(int op, int64_t M, int64_t N, int64_t K);

/* Weight quantisation and packing (Section 2, "Weight Quantization": absmean
 * to ternary; Section 5.1: packing).  Offline step, not on the timed path.
 *   W        device, in_kind 0: fp32 [N][K] row-major latent weights (beta is
 *            computed and written); in_kind 1: int8 [N][K] values in {-1,0,1}
 *            (beta is read, not written).
 *   packed   device out, bl_packed_bytes(N,K,layout) bytes.
 *   beta     device, 1 float.
 *   workspace device, bl_workspace_bytes(BL_OP_PACK, 0, N, K) bytes.
 * Enqueues three kernels (partial |W| sums in fp64, fixed-order final sum,
 * ternarize+pack).  The fp64 sum order is fixed, so beta is reproducible. */
bl_status bl_pack_ternary(const void* W, int in_kind, int64_t N, int64_t K, int layout,
                          uint8_t* packed, float* beta, void* workspace, bl_stream s);

/* Inverse of the packing, for round-trip tests: writes Wt int8 [N][K] row-major
 * in {-1,0,1} and sets *bad (device int32, zeroed by this call) to the number
 * of 2-bit fields holding the invalid code 3 (those decode to +2). */
bl_status bl_unpack_ternary(const uint8_t* packed, int64_t N, int64_t K, int layout,
                            int8_t* Wt, int32_t* bad, bl_stream s);

/* Per-token absmax int8 activation quantisation (Section 2, "Activation
 * Quantization").
 *   X      device bf16 [M][K] row-major (raw 16-bit patterns), 16-byte aligned
 *          (2-byte aligned is enough when K % 64 != 0).
 *   q      device out int8 [M][Kp], zeros in the padding;
 *   scale  device out fp32 [M] (= max(gamma,1e-5)/127);
 *   rowsum device out int32 [M], may be NULL.          M >= 1. */
bl_status bl_quant_act_int8(const uint16_t* X, int64_t M, int64_t K,
                            int8_t* q, float* scale, int32_t* rowsum, bl_stream s);

/* W1.58A8 product for decode batches, 1 <= M <= 64 (Section 5.1).  Streams the
 * packed weights once per call.
 *   packed/beta/layout  as written by bl_pack_ternary.
 *   q      device int8 [M][Kp];  scale device fp32 [M] (needed only if y != NULL).
 *   rowsum device int32 [M] or NULL (this call derives what it needs from q).
 *   acc    device out int32 [M][N] or NULL;  y device out fp32 [M][N] or NULL;
 *          at least one of the two must be non-NULL.
 *   workspace needed only when K > 8192 and rowsum is NULL (such rows go through the
 *          prefill kernel, which then computes the row sums there:
 *          bl_workspace_bytes(BL_OP_GEMV, M, N, K) bytes; BL_ERR_WORKSPACE if NULL);
 *          otherwise unused and may be NULL. */
bl_status bl_gemv_w158a8(const uint8_t* packed, const float* beta, int layout,
                         const int8_t* q, const float* scale, const int32_t* rowsum,
                         int64_t M, int64_t N, int64_t K,
                         int32_t* acc, float* y, void* workspace, bl_stream s);

/* W1.58A8 product for prefill, any M >= 1 (Section 5.1): packed tiles are
 * unpacked to int8 on chip and contracted on the int8 matrix cores.  Same
 * arguments as bl_gemv_w158a8.  If rowsum is NULL the call computes the row
 * sums itself into `workspace` (bl_workspace_bytes(BL_OP_GEMM, M, N, K) bytes,
 * then required). */
bl_status bl_gemm_w158a8(const uint8_t* packed, const float* beta, int layout,
                         const int8_t* q, const float* scale, const int32_t* rowsum,
                         int64_t M, int64_t N, int64_t K,
                         int32_t* acc, float* y, void* workspace, bl_stream s);

/* Fused BitLinear for decode, 1 <= M <= 16, K <= 8192, K % 64 == 0, M*(K+16) <= 96 KiB: the per-token absmax
 * int8 quantiser (Section 2) runs inside the product kernel (Section 5.1), so
 * one launch takes bf16 activations to fp32 outputs.  Same arithmetic, bit for
 * bit, as bl_quant_act_int8 followed by bl_gemv_w158a8.
 *   X         device bf16 [M][K].
 *   acc / y   device out [M][N], either may be NULL (not both).
 *   q_out     device out int8 [M][K] or NULL: the quantised activations;
 *   scale_out device out fp32 [M] or NULL: max(absmax,1e-5)/127 per token. */
bl_status bl_bitlinear_decode(const uint8_t* packed, const float* beta, int layout,
                              const uint16_t* X, int64_t M, int64_t N, int64_t K,
                              int32_t* acc, float* y, int8_t* q_out, float* scale_out, bl_stream s);

/* Fused producer: the elementwise step that yields the bf16 input X[m][k] of a
 * BitLinear, evaluated inside the kernel that quantises it (no bf16 tensor in
 * HBM).  Each kind is exact elementwise fp32 work, then round-to-nearest-even
 * narrowing to bf16; the quantiser then runs on those bf16 values as usual.
 *   BL_PROD_BF16       X = in0 (bf16 [M][K]).
 *   BL_PROD_F32        X = bf16(in0)                      in0 fp32 [M][K].
 *   BL_PROD_ATTN_V     context-length-1 attention over a fused QKV row
 *                      in0 fp32 [M][(n_q+2*n_kv)*head_dim] = [Q | K | V]:
 *                      X[m][h*head_dim+d] = bf16(V[m][h/(n_q/n_kv)][d]); K = n_q*head_dim.
 *   BL_PROD_RESIDUAL   t = in0 + in1 (fp32 [M][K] each), X = bf16(t); if aux_out
 *                      is given, t is also stored there (fp32 [M][K]).
 *   BL_PROD_RELU2_GATE in0 fp32 [M][2K] = [g | u]: X = bf16((max(g,0)*max(g,0))*u)
 *                      (the squared-ReLU gated FFN activation, Section 2).
 * norm != 0 adds the sub-layer normalisation in front of the quantiser (Section 2,
 * "Normalization"; the report names the scheme but gives no formula, so this is the
 * bias-free RMS form): with t[k] the fp32 value of the kind above BEFORE narrowing,
 *   ss = sum_k t[k]^2 with exact fp64 squares and an fp64 sum (relative error of the sum
 *        far below 1e-12; the order inside a kernel is fixed, so a result is reproducible),
 *   r = fp32(1 / sqrt(ss/K + eps)) in fp64,   X[k] = bf16((t[k]*r)*gain[k])
 * (gain NULL: no second multiply).  Every later step is a single rounded IEEE operation; r can
 * depend on the summation order only when 1/sqrt(ss/K+eps) lies within ~1e-12 (relative) of
 * an fp32 rounding midpoint.  BL_PROD_RESIDUAL still stores the
 * un-normalised sum in aux_out.
 * All pointers are device pointers, 16-byte aligned. */
enum { BL_PROD_BF16 = 0, BL_PROD_F32 = 1, BL_PROD_ATTN_V = 2, BL_PROD_RESIDUAL = 3, BL_PROD_RELU2_GATE = 4 };
typedef struct {
    int kind;
    const void* in0;
    const float* in1;
    float* aux_out;
    int n_q, n_kv, head_dim;
    int norm;               /* 0: none; 1: RMS normalisation as above */
    const float* gain;      /* fp32 [K] or NULL */
    float eps;              /* added to the mean square (fp32) */
} bl_producer;

/* One decode product of a group.  Give either X (bf16, fused quantiser), a
 * producer (prod.in0 != NULL, fused producer + quantiser), or q (+ scale if y is
 * wanted, + optional rowsum).  All pointers are device pointers; the descriptor
 * array itself is HOST memory, read during the call.
 * fixed_scale > 0 (fused paths only) replaces absmax/127 in the rescale, i.e.
 * the layer then acts on x/absmax (a normalised input); 0 = normal.
 * residual (fp32 [M][N] or NULL): y = residual + acc*(beta*scale), one fp32 add. */
typedef struct {
    const uint8_t* packed;
    const float* beta;
    const uint16_t* X;
    const int8_t* q;
    const float* scale;
    const int32_t* rowsum;
    int64_t N, K;
    int32_t* acc;
    float* y;
    int8_t* q_out;
    float* scale_out;
    float fixed_scale;
    bl_producer prod;
    const float* residual;
} bl_decode_desc;

/* Up to four INDEPENDENT decode products (same M, same layout, K <= 8192 each)
 * in one kernel launch, e.g. the four BitLinear shapes of a layer on
 * independent inputs.  Results are identical to separate calls; the point is
 * one launch and one continuous weight stream instead of four.
 * Limits: a product with a fused input (X or prod) needs M <= 16, K % 64 == 0 and
 * M*(K+16) <= 96 KiB; a product with int8 input (q, [M][Kp]) takes M <= 64 and any K.
 * Errors: BL_ERR_SHAPE outside these limits or for count outside 1..4. */
bl_status bl_bitlinear_decode_group(const bl_decode_desc* descs, int count, int layout, int64_t M, bl_stream s);

/* Producer + per-token absmax int8 quantiser for prefill (Section 2): like
 * bl_quant_act_int8, but the bf16 activations come from `prod` (HOST pointer to
 * the descriptor; its tensors are device memory).  One workgroup per token.
 * Needs K % 64 == 0 (BL_ERR_SHAPE otherwise). */
bl_status bl_quant_act_ex(const bl_producer* prod, int64_t M, int64_t K,
                          int8_t* q, float* scale, int32_t* rowsum, bl_stream s);

/* bl_gemm_w158a8 with an optional residual (fp32 [M][N] or NULL) added in the
 * epilogue: y = residual + acc*(beta*scale[m]), one fp32 add per element. */
bl_status bl_gemm_w158a8_res(const uint8_t* packed, const float* beta, int layout,
                             const int8_t* q, const float* scale, const int32_t* rowsum,
                             int64_t M, int64_t N, int64_t K, const float* residual,
                             int32_t* acc, float* y, void* workspace, bl_stream s);

/* Prefill product with a FUSED PRODUCER EPILOGUE (Section 2: per-token absmax activation
 * quantisation, ReLU^2 in the FFN): the elementwise step that turns this product's output into
 * the next BitLinear's input runs in the product's epilogue, so the fp32 output is not written
 * and read again just to be narrowed.  The epilogue writes the bf16 input of the next BitLinear
 * and folds the row maximum of its absolute values into absmax[] (an order-free maximum on the
 * float bits, across all workgroups of the launch); bl_quant_from_absmax then quantises in one
 * pass.  Bit for bit the same numbers as bl_gemm_w158a8[_res] followed by bl_quant_act_ex.
 *   BL_EPI_RESIDUAL    t = residual[m][n] + acc*(beta*scale[m]);  N_out = N
 *   BL_EPI_RELU2_GATE  the matrix is a fused [gate | up] pair (rows n and N/2 + n):
 *                      g = acc_g*(beta*scale[m]), u = acc_u*(..), t = (max(g,0)*max(g,0))*u;
 *                      N_out = N/2; needs N % 128 == 0
 *   y       device out fp32 [M][N_out] or NULL: t itself (wanted when t is a later residual)
 *   x_bf16  device out bf16 [M][N_out]: bf16(t)
 *   absmax  device in/out fp32 [M]: must hold 0 (or an earlier partial maximum of the same rows)
 *           before the launch; receives max_n |bf16(t)|.  bl_quant_from_absmax clears it again.
 *   acc     device out int32 [M][N] or NULL (the raw accumulators, natural column order).
 * Needs layout BL_LAYOUT_K16, K % 128 == 0 and rowsum (BL_ERR_LAYOUT / BL_ERR_SHAPE / BL_ERR_NULL). */
enum { BL_EPI_RESIDUAL = 1, BL_EPI_RELU2_GATE = 2 };
typedef struct {
    int kind;
    const float* residual;   /* BL_EPI_RESIDUAL: fp32 [M][N] */
    float* y;
    uint16_t* x_bf16;
    float* absmax;
} bl_gemm_epilogue;
bl_status bl_gemm_w158a8_fused(const uint8_t* packed, const float* beta, int layout,
                               const int8_t* q, const float* scale, const int32_t* rowsum,
                               int64_t M, int64_t N, int64_t K, const bl_gemm_epilogue* ep /* HOST */,
                               int32_t* acc, bl_stream s);
/* One-pass quantiser for rows whose absmax is already known: like bl_quant_act_int8 with
 * gamma = absmax[m] given; clears absmax[m] to 0 afterwards.  Needs K % 64 == 0. */
bl_status bl_quant_from_absmax(const uint16_t* X, float* absmax, int64_t M, int64_t K,
                               int8_t* q, float* scale, int32_t* rowsum, bl_stream s);

/* Persistent streaming decode over a TABLE of products (Section 5.1: the decode kernel is
 * there to use as little memory bandwidth as possible, which on this GPU means the weight
 * stream of a whole stack of BitLinears must never stop).  One launch walks every product
 * of the table with as many workgroups as stay resident; each product is the same
 * arithmetic, bit for bit, as one entry of bl_bitlinear_decode_group.  Entries with a fused
 * input are quantised (Section 2) without a pass of their own: a plain bf16 input (X) inside
 * the stream launch, by each workgroup that meets the product (about five hundred workgroups
 * over the table, each meeting one or two products; no data crosses workgroups); a
 * producer or a normalised input (prod) by a small preparation launch in front of it (one
 * workgroup per such entry, into scratch inside `table`; the same launch computes a missing
 * rowsum of an int8 entry); int8 entries are streamed as they are.
 * The products of one table are INDEPENDENT: none may read what another writes.
 * Entries with a fused input need K % 64 == 0; int8 entries (q of Kp bytes) take any K.
 *   bl_stack_table_bytes  device bytes `table` needs for these descriptors (HOST array): the
 *                         table itself plus the scratch for quantised rows.  0: bad count or K.
 *   bl_stack_build        setup call: checks the descriptors (HOST array), lays the work out
 *                         over the grid, copies the table to `table` (device, 256-byte
 *                         aligned, caller-owned) and fills *plan (HOST, caller-owned).  It
 *                         waits for that copy on `s` (the only call here that synchronises).
 *                         Limits: 1 <= count <= 1024; M = 1: K <= 20480 per product (M > 1:
 *                         the batched form below).
 *   bl_stack_run          at most two kernel launches on `s` (preparation, stream); no
 *                         allocation, no synchronisation; may be captured in a HIP graph and
 *                         replayed.  The table and every tensor it names must stay alive and
 *                         in place; runs on one table must not overlap (they share the scratch).
 * BATCHED FORM, 2 <= M <= BL_STACK_MAX_TOKENS tokens per product (batched decode: the weights
 * of the table are still read once per run): bl_stack_build with M > 1 takes int8 entries only
 * (q [M][Kp], scale [M] when y is wanted, rowsum [M]; outputs [M][N]; BL_ERR_VALUE for X / prod,
 * BL_ERR_NULL without rowsum), layout BL_LAYOUT_K16 (BL_ERR_LAYOUT otherwise), any N and K;
 * `table` needs bl_stack_table_bytes_batched bytes (0: bad count, M, N or K).  The kernel keeps
 * the token rows of a table entry in LDS and multiplies on the matrix cores, 32 tokens to a tile.
 * How a product becomes table entries is the library's business and never changes a result:
 * up to 64 tokens in one entry where their rows fit LDS whole, else groups of at most 32 tokens
 * (the weights are then read once per group); rows too long for LDS are cut into k parts whose
 * partial sums meet in scratch inside `table` through integer atomics (exact, order-free) and
 * are finished (row sum, rescale, residual) by a second small launch of the same run, which
 * also clears the scratch.  plan->entries tells how many entries the table holds.
 * With more than 48 tokens, and every row length a multiple of 128 after padding, the table is
 * walked by the prefill tile kernel instead (Section 5.1: packed tiles expanded to int8 on chip
 * for the int8 matrix cores): 64 x 128 output tiles, both operands streamed through LDS, the
 * tiles of all products balanced over the resident workgroups by their k steps, one launch,
 * weights read once; plan->red_ints then holds the tile count.
 * Same arithmetic, bit for bit, as bl_gemv_w158a8 on each product. */
enum { BL_STACK_MAX_COUNT = 1024, BL_STACK_MAX_TOKENS = 64 };
typedef struct {
    int32_t count, blocks, prep_count, inline_count, norm, lds_bytes, layout, red_ints;
    int64_t wg_offset, prep_offset;   /* byte offsets inside `table`                            */
    int64_t packed_bytes;             /* packed weight bytes of the products: what one run streams */
    int64_t table_bytes;
    int32_t tokens, entries;          /* M; table entries (> count when products were split)    */
} bl_stack_plan;
size_t    bl_stack_table_bytes(const bl_decode_desc* descs, int count);
size_t    bl_stack_table_bytes_batched(const bl_decode_desc* descs, int count, int64_t M);
bl_status bl_stack_build(const bl_decode_desc* descs, int count, int layout, int64_t M,
                         void* table, bl_stack_plan* plan, bl_stream s);
bl_status bl_stack_run(void* table, const bl_stack_plan* plan, bl_stream s);

/* bl_gemm_w158a8 for callers that cannot allocate device memory or bring a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same product and same results as bl_gemm_w158a8 called with rowsum = NULL;
 * the scratch for the row sums sum_k q[m][k] is a static device array inside the library
 * (64 KiB per GPU, held until the process ends), so the call allocates and frees nothing.
 * Limit: 1 <= M <= 16384, else BL_ERR_SHAPE.  All calls on one GPU share that array:
 * calls that overlap on the same GPU (different streams or threads) race; calls on one
 * stream, or otherwise ordered, are safe.  Nothing needs clearing between calls. */
bl_status bl_gemm_w158a8_noalloc(const uint8_t* packed, const float* beta, int layout,
                                 const int8_t* q, const float* scale,
                                 int64_t M, int64_t N, int64_t K,
                                 int32_t* acc, float* y, bl_stream s);

/* Test hook: which decode kernel the M <= 64 entry points take, so that tests can put every
 * kernel through every case.  0 = the measured default, 1 = the dot4 kernel where it applies
 * (M <= 4), 2 = the row-resident matrix-core kernel, 3 = the streaming panel kernel where it
 * applies (int8 inputs).  Process-wide and atomic; results never depend on it, only the route.
 * BL_ERR_VALUE outside 0..3. */
bl_status bl_debug_force_path(int path);

/* Measurement aids (not part of the product path): the achievable roofs the kernels are
 * priced against beside the datasheet peaks.
 *   bl_probe_stream_read  one launch that reads `bytes` (a multiple of 16) of device memory
 *                         at `buf` with 128-bit loads and does nothing else; time it over a
 *                         buffer much larger than the caches to get the streaming-read rate.
 *                         workgroups_per_cu: 256-thread workgroups per compute unit, 1..8
 *                         (0 = 8, the fastest); 2 is the occupancy of the streaming decode.
 *   bl_probe_stream_write one launch that fills a row-major fp32 matrix [rows][cols] (device, both
 *                         multiples of 128) with the store pattern of the prefill epilogue (128 x 128
 *                         tiles, dword stores of 32 consecutive floats per row, non-temporal) and
 *                         does nothing else: the rate at which the outputs of a prefill launch can be
 *                         written when every workgroup stores at once.  workgroups_per_cu 1..8
 *                         (0 = 3, the occupancy of the tile kernel).
 *   bl_probe_mfma_i8      one launch of `iters` x 4 back-to-back v_mfma_i32_32x32x32_i8 per
 *                         wave, operands in registers; *ops (HOST, optional) receives the
 *                         integer operations of the launch (2 per multiply-accumulate).
 *   bl_probe_mfma_i8_ex   the same loop with its operands read once from `operands` (device,
 *                         64 KiB of int8, or NULL for the constants of bl_probe_mfma_i8): with
 *                         random operands the loop draws more power and the chip runs it at a
 *                         lower clock, which is the rate a real contraction can hope for.
 *                         stamps (device, 2 x int64, or NULL) receives what workgroup 0 counted
 *                         between its first and last instruction: [0] shader clocks, [1] ticks of
 *                         the constant-rate wall clock (bl_probe_wall_clock_khz), so
 *                         stamps[0] / stamps[1] x that rate is the clock the kernel ran at.
 *   bl_probe_wall_clock_khz  rate of that wall clock in kHz (0 on error).  Host-only query.
 *   bl_debug_clock_stamps  measurement hook for the prefill tile kernel: while a device buffer
 *                         of 2 x int64 is registered, every launch of that kernel (bl_gemm_w158a8
 *                         and its variants on the direct-to-LDS path) leaves the same two counts
 *                         of its workgroup 0 there; NULL (the default) switches it off.
 *                         Process-wide and atomic; results never depend on it.
 * sink: device, 64 int32, never written in practice (it keeps the work observable). */
bl_status bl_probe_stream_read(const void* buf, size_t bytes, int workgroups_per_cu, int32_t* sink,
                               bl_stream s);
bl_status bl_probe_stream_write(float* buf, int64_t rows, int64_t cols, int workgroups_per_cu, bl_stream s);
bl_status bl_probe_mfma_i8(int iters, int32_t* sink, double* ops, bl_stream s);
bl_status bl_probe_mfma_i8_ex(int iters, const void* operands, int64_t* stamps, int32_t* sink, double* ops /* HOST */,
                              bl_stream s);
int       bl_probe_wall_clock_khz(void);
bl_status bl_debug_clock_stamps(int64_t* stamps);

#ifdef __cplusplus
}
#endif
#endif /* BITLINEAR_H */
