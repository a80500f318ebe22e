/*
 * nm.h -- C ABI of libnm: N:M-sparse, low-bit-integer linear layers on MI355X (gfx950).
 *
 * Naming: N = weights kept per group, M = group width, groups run along the
 * input (reduction) dimension.  The paper writes the same pattern the other way
 * round ("4:2" there is N=2, M=4 here).
 *
 * Ownership and execution model (all entry points):
 *   - every *_dev pointer is DEVICE memory owned by the caller; the library
 *     allocates nothing and never frees anything; the only device memory of its
 *     own is the fixed scratch array of nm_scale_search_static (see there), and no
 *     result depends on anything an earlier call left behind;
 *   - work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns without synchronising;
 *   - buffers of one call must not overlap;
 *   - arguments are validated on the host before anything is launched; a
 *     negative return value means nothing was enqueued.
 */
#ifndef NM_H
#define NM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum nm_status {
    NM_OK = 0,
    NM_ERR_NULL = -1,     /* a required pointer is NULL                                   */
    NM_ERR_DIM = -2,      /* rows/cols/tokens <= 0 or a leading dimension below its extent */
    NM_ERR_PATTERN = -3,  /* M not in {4, 8}, N < 1, N > M, cols % M != 0, or (tiled layout)
                             cols % 128 != 0                                               */
    NM_ERR_BITS = -4,     /* bits not in {4, 8}                                            */
    NM_ERR_DTYPE = -5,    /* unknown output dtype, or dtype set with a NULL output         */
    NM_ERR_ALIGN = -6,    /* pointer or leading dimension violates a stated alignment      */
    NM_ERR_HIP = -7,      /* the HIP runtime reported an error at launch                   */
    NM_ERR_LAYOUT = -8,   /* unknown layout code                                           */
    NM_ERR_SCALE = -9,    /* a host-side scale that is not a positive finite number        */
    NM_ERR_WORKSPACE = -10 /* a workspace smaller than its size query asks for             */
};

/*
 * Layout of the packed values and of the index metadata in memory (the paper never discusses
 * one; both are this library's definitions).  The same bytes either way: the tiled layout is a
 * permutation of the row layout, fixed below, and every entry point takes either.
 */
enum nm_layout {
    NM_LAYOUT_ROWS = 0,   /* one packed row after the other: the interchange format          */
    NM_LAYOUT_TILED = 1   /* what one matrix-core fragment consumes (16 rows x 128 input
                             columns) is one contiguous run of memory: the format the fast
                             nm_gemm kernels read; needs cols % 128 == 0                     */
};

enum nm_out_dtype {
    NM_OUT_NONE = 0,      /* no dequantised output (accumulators only)   */
    NM_OUT_F32 = 1,       /* float                                       */
    NM_OUT_BF16 = 2       /* bfloat16, round-to-nearest-even from float  */
};

/*
 * Byte sizes of the three packed buffers of a rows x cols matrix (host only, no
 * GPU needed).  Any of the three out-pointers may be NULL.
 *
 * Row layout.  kc = cols*N/M kept entries per row, entry e = g*N + j is the j-th kept column
 * (ascending) of group g.
 *   values : row-major, row stride ceil(kc*bits/8) bytes; bits=8: entry e is byte e;
 *            bits=4: two's-complement nibbles, entry e in byte e/2, low nibble for
 *            even e, high nibble for odd e.
 *   meta   : row-major, row stride ceil(kc*ib/8) bytes, ib = 2 for M=4 and 4 for
 *            M=8; entry e's column offset inside its group occupies ib bits at bit
 *            e*ib of the row, LSB-first through the bytes.
 *   scales : float[rows].
 * Unused trailing bits of a row are zero.  A dense matrix (N = M: every entry kept, the
 * 8-bit / 4-bit components without sparsity of Sec. 5.4) has no metadata: meta_bytes = 0,
 * meta_dev may be NULL, entry e is column e.
 *
 * Tiled layout (cols % 128 == 0).  A unit is the packed bytes of one row that cover 32
 * consecutive input columns: unit u of row r is bytes [u*UB, (u+1)*UB) of row r in the row
 * layout, with UB = (32/M)*N*bits/8 for the values and (32/M)*N*ib/8 for the metadata.  The 64
 * units of 16 consecutive rows (row block rb = r/16) and one 128-column slice (s = u/4) form
 * block (rb, s), which starts at byte (rb*(cols/128) + s)*64*UB of the buffer; rows are padded
 * with zero bytes up to a multiple of 16.  Inside a block unit number j = (u%4)*16 + r%16; a
 * unit is cut into pieces of PB bytes, PB the largest power of two <= 16 that divides UB, and
 * piece p of unit j lies at byte (p*64 + j)*PB of the block.  (For 2:4 int8 a block is the
 * A-operand of the sparse 16x16x128 integer MFMA in lane order, 16 bytes per lane.)  The
 * scales are float[rows] as in the row layout.
 */
int nm_packed_sizes(int rows, int cols, int N, int M, int bits, int layout,
                    size_t *vals_bytes, size_t *meta_bytes, size_t *scales_bytes);

/*
 * Constrain a trained fp32 matrix to N:M sparsity and `bits`-bit symmetric
 * integers and pack it: the projection of Sec. 3.2 (Eq. 3: keep the N
 * largest-magnitude entries of every M-wide group) followed by the max-rule scale
 * of Sec. 3.3.1 and the quantiser of Sec. 3.3 (Eq. 5, offset 0), applied directly
 * to the given weights as in Sec. 4.
 *
 *   W_dev      [rows][ldw] float, row-major; rows = output neurons, cols = inputs;
 *              ldw (elements) >= cols; 4-byte aligned (NM_ERR_ALIGN otherwise).  With W_dev
 *              and ldw*4 16-byte aligned, vals_dev / meta_dev 4-byte aligned and packed rows
 *              that are whole dwords the wavefront-per-row kernels run; anything else takes
 *              a slow thread-per-row kernel, same bytes.
 *   layout     nm_layout of the outputs.
 *   vals_dev, meta_dev, scales_dev   outputs, sizes from nm_packed_sizes; scales_dev 4-byte
 *              aligned; meta_dev may be NULL for a dense matrix.
 *
 * Definitions the paper leaves open: equal magnitudes keep the lower column; one
 * scale per row, s = max|w| / (2^(bits-1)-1) with an all-zero row giving s = 1;
 * code = clamp(rne(w / s), -(2^(bits-1)-1), +(2^(bits-1)-1)) using IEEE fp32
 * divisions and round-half-to-even.  Non-finite weights give unspecified bytes.
 */
int nm_compress(const float *W_dev, int rows, int cols, int ldw,
                int N, int M, int bits, int layout,
                void *vals_dev, void *meta_dev, float *scales_dev,
                void *hip_stream);

/*
 * The same with one scale per group of rows_per_scale consecutive output neurons (Sec. 3.3:
 * group-wise quantisation, parameters of one neuron always sharing a scale; Sec. 4: 32 neurons
 * per scale is the paper's default): s = (largest |w| over the rows of the group) /
 * (2^(bits-1)-1), 1 for an all-zero group; the last group may be shorter.  The packed format is
 * unchanged - scales_dev still receives one float per row, the rows of a group holding the same
 * value - so nm_gemm and nm_decompress_i8 take the result as it is.  rows_per_scale = 1 is
 * nm_compress.  scales_dev also serves as the call's scratch space.
 */
int nm_compress_grouped(const float *W_dev, int rows, int cols, int ldw,
                        int N, int M, int bits, int layout, int rows_per_scale,
                        void *vals_dev, void *meta_dev, float *scales_dev,
                        void *hip_stream);

/*
 * The paper's second scale rule (Sec. 3.3.1, "ADMM-Dist": choose the scale that minimises the L2
 * distance between the quantised and the raw parameters), per group of rows_per_scale consecutive
 * output neurons.  The paper states the criterion, not an algorithm; the library searches a grid:
 *
 *   s_max   the max-rule scale of the group (largest |w| / (2^(bits-1)-1), 1 for an all-zero group)
 *   s_c     = (s_max * c) / candidates for c = candidates/2 .. candidates   (fp32: a multiplication,
 *             then a division): from the max rule itself down to half of it
 *   err(c)  = sum over the entries the N:M projection keeps (as nm_compress keeps them) of
 *             (w - s_c * q)^2 with q = clamp(rne(w / s_c)), formed and summed in double
 *   scale   = the s_c of least error; between equal errors the larger scale
 *
 * scales_dev[rows] receives every row's scale (the rows of a group hold the same value), ready
 * for nm_compress_scaled.  Errors are summed in a fixed order that is not the plain left-to-right
 * one, so two candidates whose errors agree to about 1e-15 relative may be ranked either way.
 *
 *   candidates      even, 2 .. 64.
 *   workspace_dev   device scratch of nm_scale_search_workspace_bytes(rows, candidates) bytes
 *                   (the rows' partial errors, [rows][candidates/2 + 1] doubles), 8-byte aligned,
 *                   owned by the caller; contents before and after the call do not matter.
 * Errors as for nm_compress_grouped; NM_ERR_WORKSPACE when workspace_bytes is too small.
 */
size_t nm_scale_search_workspace_bytes(int rows, int candidates);

int nm_scale_search(const float *W_dev, int rows, int cols, int ldw,
                    int N, int M, int bits, int rows_per_scale, int candidates,
                    float *scales_dev, void *workspace_dev, size_t workspace_bytes,
                    void *hip_stream);

/*
 * nm_scale_search for callers that cannot allocate or pass device memory of their own for scratch:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * launches, the same result bit for bit; the rows' partial errors go to an array built into the
 * library (static device memory, NM_SCALE_SEARCH_STATIC_MAX_BYTES per GPU, held from the first call
 * on that GPU until the process ends) instead of a workspace.  The call allocates and frees
 * nothing.
 *   - rows * (candidates/2 + 1) * 8 must not exceed NM_SCALE_SEARCH_STATIC_MAX_BYTES (3072 rows at
 *     64 candidates need 0.8 MB): NM_ERR_WORKSPACE otherwise, with a message on stderr, nothing
 *     enqueued; larger problems take nm_scale_search.
 *   - every call on a GPU uses that GPU's one array: calls that overlap in time on the same GPU
 *     (different streams without an ordering between them) race on it and give wrong scales.
 *     Nothing in the array has to be cleared between calls.
 *   - the first call on a GPU looks the array's address up (hipGetSymbolAddress, once per device);
 *     make that call outside any stream capture.
 * Other arguments and errors as for nm_scale_search.
 */
#define NM_SCALE_SEARCH_STATIC_MAX_BYTES (2u << 20)
int nm_scale_search_static(const float *W_dev, int rows, int cols, int ldw,
                           int N, int M, int bits, int rows_per_scale, int candidates,
                           float *scales_dev, void *hip_stream);

/*
 * nm_compress with the scales given: scales_dev[rows] is an INPUT (one scale per row, each a
 * positive finite float: those of nm_scale_search, or a caller's own), everything else as
 * nm_compress - same projection, same quantiser, same packed formats.
 */
int nm_compress_scaled(const float *W_dev, int rows, int cols, int ldw,
                       int N, int M, int bits, int layout, const float *scales_dev,
                       void *vals_dev, void *meta_dev, void *hip_stream);

/*
 * nm_compress on several matrices of one pattern in one call - the weight matrices of an encoder
 * layer, say (Sec. 4 compresses every linear layer of the encoder the same way).  Item i gives
 * exactly what nm_compress(items[i].W_dev, rows, cols, ldw, N, M, bits, layout, vals_dev,
 * meta_dev, scales_dev) gives, byte for byte; the matrices that meet nm_compress's alignment share launches
 * (the fixed cost of a launch is several times the time their bytes take), the others go one by
 * one.  `items` is HOST memory, read during the call and not kept; the device buffers of
 * different items must not overlap; count <= 0 or count > NM_COMPRESS_BATCH_MAX_ITEMS is an error
 * (NM_ERR_DIM), as is any item nm_compress would refuse (then nothing is enqueued).
 */
#define NM_COMPRESS_BATCH_MAX_ITEMS 65536
typedef struct nm_compress_item {
    const float *W_dev;   /* [rows][ldw] float                        */
    int rows, cols, ldw;
    void *vals_dev;       /* outputs, sizes from nm_packed_sizes      */
    void *meta_dev;
    float *scales_dev;
} nm_compress_item;

int nm_compress_batch(const nm_compress_item *items, int count,
                      int N, int M, int bits, int layout, void *hip_stream);

/*
 * The packed values and metadata of a matrix from one layout to the other (layout_in names the
 * layout of the inputs; the outputs are in the other one, sizes from nm_packed_sizes): for weights
 * that were compressed, stored or exchanged in the row layout and are to be multiplied by the
 * fast kernels, which read the tiled one.  A pure byte permutation (the padding rows of the tiled
 * layout are written as zeros); the scales are layout-independent and not touched.  Needs
 * cols % 128 == 0; the buffers must not overlap.
 */
int nm_repack(const void *vals_in_dev, const void *meta_in_dev, int rows, int cols,
              int N, int M, int bits, int layout_in,
              void *vals_out_dev, void *meta_out_dev, void *hip_stream);

/*
 * Expand packed weights to the dense integer matrix Wq_dev[rows][cols] (int8,
 * zeros at pruned positions, int4 codes sign-extended).  Inverse of the packing
 * step; used to check that the sparse product equals the dense one.
 */
int nm_decompress_i8(const void *vals_dev, const void *meta_dev, int rows, int cols,
                     int N, int M, int bits, int layout, int8_t *Wq_dev, void *hip_stream);

/*
 * The sparse integer linear layer of Sec. 5.3 with the dequantisation of Sec. 3.3
 * (Eq. 4, offset 0) fused behind it:
 *
 *   acc[t][o] = sum over kept entries e of row o:  X[t][col(o,e)] * q[o][e]   (int32, exact)
 *   y[t][o]   = float(acc[t][o]) * (act_scale * scales[o])  (+ bias[o])
 *
 *   X_dev      [tokens][ldx] int8 activations, ldx >= K.
 *   act_scale  per-tensor activation scale (host value).
 *   act_scale_dev   NULL, or one device float that replaces act_scale and is read when the
 *              kernel runs (see nm_gemm_q8).
 *   vals_dev, meta_dev, scales_dev   packed weights of an O x K matrix as written by
 *              nm_compress with the same N, M, bits, layout.
 *   bias_dev   float[O] or NULL.
 *   acc_dev    int32 [tokens][ldo] or NULL (exact accumulators, optional).
 *   out_dev    [tokens][ldo] of out_dtype, or NULL with NM_OUT_NONE.
 *   ldo        leading dimension (elements) of acc_dev and out_dev, >= O.
 *
 * At least one of acc_dev / out_dev must be given.  Low-bit weights are widened to
 * int8 in registers; products of pruned positions are never formed on the 2:4
 * hardware path.  Results do not depend on launch shape (integer sums are exact;
 * the epilogue is elementwise).
 *
 * Alignment.  Required (NM_ERR_ALIGN): scales_dev, bias_dev, acc_dev 4-byte aligned, out_dev
 * aligned to its element.  The matrix-core kernels additionally need K % 128 == 0, O % 4 == 0,
 * ldo % 4 == 0 and 16-byte aligned X_dev, ldx, vals_dev, meta_dev, scales_dev, bias_dev, acc_dev,
 * out_dev, and a pattern they cover: N <= 2 (either layout; the tiled layout runs the fastest
 * kernels), or any other pattern (N >= 3, dense N = M included) in the tiled layout.  Any other
 * call is computed by a slow one-thread-per-output kernel with the same results.
 */
int nm_gemm(const int8_t *X_dev, int tokens, int K, int ldx, float act_scale,
            const float *act_scale_dev,
            const void *vals_dev, const void *meta_dev, const float *scales_dev,
            int O, int N, int M, int bits, int layout,
            const float *bias_dev,
            int32_t *acc_dev,
            void *out_dev, int out_dtype,
            int ldo, void *hip_stream);

/*
 * Several linear layers of one scheme in one launch: the query, key and value layers of an
 * attention block, say, where the chosen configuration compresses them alike (Sec. 5.4 lists the
 * three as separate components; Sec. 5.3's GEMMs otherwise).  Item i gives exactly what
 * nm_gemm(items[i].X_dev, ..., N, M, bits, layout, ..., out_dtype, items[i].ldo) gives, element
 * for element; N, M, bits, layout and out_dtype are common to all items, every other argument
 * is per item with nm_gemm's meaning, requirements and errors (shapes and inputs may differ
 * between items; several items may read the same X_dev).  Where every item meets what
 * nm_gemm's matrix-core kernels need in the tiled layout, the items' output tiles are computed
 * by one kernel launch (each launch costs about two microseconds of idle time between kernels,
 * a third of such a layer's GEMM at 4096 tokens); otherwise the items are launched one after the
 * other.  `items` is HOST memory, read during the call and not kept; the output buffers of
 * different items must not overlap each other or any input.  count <= 0 or
 * count > NM_GEMM_BATCH_MAX_ITEMS is NM_ERR_DIM; an item nm_gemm would refuse gives its error
 * and nothing is enqueued.
 */
#define NM_GEMM_BATCH_MAX_ITEMS 4
typedef struct nm_gemm_item {
    const int8_t *X_dev;          /* [tokens][ldx] int8                                   */
    int tokens, K, ldx;
    float act_scale;
    const float *act_scale_dev;   /* replaces act_scale when not NULL                     */
    const void *vals_dev;         /* packed weights of an [O][K] matrix                   */
    const void *meta_dev;
    const float *scales_dev;      /* float[O]                                             */
    int O;
    const float *bias_dev;        /* float[O] or NULL                                     */
    int32_t *acc_dev;             /* [tokens][ldo] or NULL                                */
    void *out_dev;                /* [tokens][ldo] of out_dtype, or NULL with NM_OUT_NONE */
    int ldo;
} nm_gemm_item;

int nm_gemm_batch(const nm_gemm_item *items, int count,
                  int N, int M, int bits, int layout, int out_dtype, void *hip_stream);

/*
 * Training side of the same constraints: the Z-update of the ADMM decomposition (Sec. 3.1),
 * Z = Pi(W + U), i.e. Eq. 3 applied to W + U, with the quantisation constraint solved after the
 * sparsity constraint (Sec. 3.3.1: in that order the two projections in sequence are the joint
 * projection; scale by the largest-parameter rule, "ADMM-Max") and one scale per group of
 * rows_per_scale consecutive output neurons (Sec. 4: 32 by default), plus the scaled dual update
 * U <- U + W - Z.  fp32 throughout, one operation per step, in this order:
 *
 *   V     = W + U                                   (U_dev NULL: V = W)
 *   keep  = the N largest |V| of every M consecutive columns; equal magnitudes: the lower column
 *   bits 0: Z = V on kept positions, +0 elsewhere   (the sparsity constraint alone)
 *   bits 4 or 8: s = (largest |V| over the rows of the scale group) / (2^(bits-1) - 1), 1 for an
 *           all-zero group; q = clamp(rne(V / s)) as in nm_compress; Z = s * q on kept
 *           positions, +0 elsewhere
 *   U_out = V - Z                                   (when U_out_dev is given)
 *
 *   W_dev, U_dev     float [rows][ldw]; U_dev may be NULL.  16-byte aligned, ldw % 4 == 0.
 *   Z_dev, U_out_dev float [rows][ldz]; U_out_dev may be NULL, and with ldz == ldw it may be U_dev
 *                    itself (every element is read before it is written, by the same thread);
 *                    Z_dev must not overlap the inputs.  16-byte aligned, ldz % 4 == 0.
 *   scales_dev       float[rows], required when bits > 0: receives every row's scale (the rows of
 *                    one group hold the same value); it also serves as the call's scratch space.
 *   rows_per_scale   >= 1; the last group may be shorter.
 * Errors as for nm_compress (bits may also be 0 here).
 */
int nm_project(const float *W_dev, const float *U_dev, int rows, int cols, int ldw,
               int N, int M, int bits, int rows_per_scale,
               float *Z_dev, float *U_out_dev, int ldz, float *scales_dev, void *hip_stream);

/*
 * The same layer with its output handed on as 8-bit activations (Sec. 5.3: activations are
 * 8-bit integers), i.e. Eq. 4 followed by the scalar quantiser of Sec. 3.3, Eq. 5 (offset 0,
 * 8 bits) with a scale the caller supplies, so that a chain of layers never writes or re-reads a
 * floating-point tensor:
 *
 *   q[t][o] = clamp(rne(y[t][o] / out_scale), -127, 127),   y as nm_gemm defines it.
 *
 * How it is evaluated.  The division is taken once per output column, folded into the column's
 * multiplier and offset, one fp32 operation per step:
 *   g[o]    = (act_scale * scales[o]) / out_scale        (multiplication, then true division)
 *   h[o]    = bias[o] / out_scale, or 0 without bias
 *   z[t][o] = fma(float(acc[t][o]), g[o], h[o]),   q = clamp(rne(z), -127, 127)   (ties to even)
 * z differs from the exactly divided y / out_scale by less than
 * 1e-6 * (|acc| * act_scale * scales[o] + |bias[o]|) / out_scale, so a code can differ (by one)
 * from the one a division per output gives only where y / out_scale lies within that distance of
 * a half-way point k + 1/2.
 *
 *   out_scale   > 0, finite (host value; NM_ERR_SCALE otherwise).
 *   act_scale_dev, out_scale_dev   NULL, or one device float each that replaces the host value
 *               of the same name and is read when the kernel runs - a scale computed on the
 *               device by earlier work on the stream (nm_absmax_to_scale), so that a captured
 *               chain of layers follows the statistics of its own activations.  A device
 *               out_scale must be positive and finite (not checked: the host cannot see it).
 *   out_dev     int8 [tokens][ldo], ldo >= O, 4-byte aligned (rows that are whole 16-byte
 *               pieces, ldo % 16 == 0 with a 16-byte aligned out_dev, are written fastest).
 *   absmax_dev  NULL, or one float that the caller has set (to 0, or to a running maximum
 *               >= 0) before the call: (max over all outputs of |z|) * out_scale, i.e. max |y|
 *               up to the rounding above, is max-combined into it atomically - the statistic
 *               from which the next out_scale is chosen.
 * Other arguments as for nm_gemm.
 */
int nm_gemm_q8(const int8_t *X_dev, int tokens, int K, int ldx, float act_scale,
               const float *act_scale_dev,
               const void *vals_dev, const void *meta_dev, const float *scales_dev,
               int O, int N, int M, int bits, int layout,
               const float *bias_dev, float out_scale, const float *out_scale_dev,
               int8_t *out_dev, int ldo, float *absmax_dev, void *hip_stream);

/*
 * The per-tensor scale of 8-bit activations from their largest magnitude (Sec. 5 keeps
 * activations at 8 bits; the rule is the one the weights use in Sec. 3.3.1): on the stream,
 * *scale_dev = *absmax_dev / 127 (one fp32 division; 1 when the maximum is 0), and then, when
 * `reset` is non-zero, *absmax_dev = 0 for the next round of nm_gemm_q8 calls.  One tiny kernel;
 * both pointers are single device floats, 4-byte aligned, and must differ.
 */
int nm_absmax_to_scale(float *absmax_dev, float *scale_dev, int reset, void *hip_stream);

/*
 * The largest magnitude of a floating-point activation tensor (the statistic of the
 * largest-magnitude rule, Sec. 3.3.1, for the 8-bit activations of Sec. 5.3): on the stream,
 * *absmax_dev = max(*absmax_dev, max over t < tokens, k < K of |X[t][k]|), combined atomically.
 * The caller sets *absmax_dev (to 0, or to a running maximum >= 0) before the call; several
 * tensors may share one statistic.  One pass that reads 4 bytes per element.
 *
 *   X_dev       fp32 [tokens][ldx], row-major, device, 4-byte aligned; read only.  Finite values
 *               (not checked: a NaN is ignored, an infinity becomes the maximum).  16-byte
 *               aligned with K % 4 == 0 and ldx % 4 == 0 (or ldx == K and tokens * K % 4 == 0)
 *               is read fastest.
 *   tokens, K   > 0; ldx >= K  (NM_ERR_DIM otherwise).
 *   absmax_dev  one device float, 4-byte aligned.
 */
int nm_absmax_f32(const float *X_dev, int tokens, int K, int ldx, float *absmax_dev, void *hip_stream);

/*
 * A floating-point activation tensor as the 8-bit integers nm_gemm takes (Sec. 5.3; the
 * quantiser is Eq. 5 of Sec. 3.3 with offset 0 at 8 bits, exactly as nm_compress applies it to
 * the weights):
 *
 *   Xq[t][k] = clamp(rne(X[t][k] / s), -127, 127),   the quotient correctly rounded in fp32,
 *
 * with one scale s for the whole tensor: `scale`, or the device float `scale_dev` when that is
 * not NULL - read when the kernel runs, e.g. what nm_absmax_to_scale wrote after nm_absmax_f32,
 * which makes s = max|X| / 127, the rule of Sec. 3.3.1.  One pass that reads 4 bytes and writes
 * 1 byte per element.  The same s is the act_scale (act_scale_dev) of the nm_gemm that follows.
 *
 *   X_dev       as for nm_absmax_f32.  Finite values (not checked; the code of a NaN is
 *               unspecified, an infinity takes the clamp's +-127).
 *   scale       > 0, finite when scale_dev is NULL (NM_ERR_SCALE otherwise); a device scale
 *               must be positive and finite too (not checked: the host cannot see it).
 *   Xq_dev      int8 [tokens][ldq], ldq >= K, device; written for k < K only.  4-byte aligned
 *               with ldq % 4 == 0 (or ldq == ldx == K) next to the alignment named for X_dev is
 *               written fastest; any other alignment takes a kernel of one element per lane.
 *   X_dev and Xq_dev must not overlap.
 */
int nm_quantize_act(const float *X_dev, int tokens, int K, int ldx, float scale, const float *scale_dev,
                    int8_t *Xq_dev, int ldq, void *hip_stream);

/* Human-readable name of a status code (static string, never NULL). */
const char *nm_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* NM_H */
