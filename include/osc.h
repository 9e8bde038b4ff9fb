/*
 * libosc -- the inference-time dual-path linear layer of OSC (outlier separation
 * in the channel dimension) for AMD MI355X (gfx950).  C ABI.
 *
 * Conventions shared by every entry point
 *   - Linear layer Y = X . W^T with X[M, K] (tokens x input channels) and
 *     W[N, K] (output x input channels).  Quantisation groups are 32 consecutive
 *     input channels (MXFP4, G = 32) unless an entry point says otherwise (scale
 *     groups of 64: OSC_FMT_MXFP4_OSC_G64, osc_pack_weight_g).
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless marked
 *     "host".  The library never allocates, frees or keeps a pointer past the call
 *     (its only device memory of its own is one static 128 KB table, see
 *     osc_swiglu_quantize_act).
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     enqueue work and return; they never synchronise the device.
 *   - Return value: OSC_OK or a negative error; on error nothing was launched.
 *     osc_last_error() gives a thread-local description of the last error.
 *   - M == 0 or N == 0 is a valid no-op.
 *   - bf16 tensors are raw 16-bit patterns.  Inputs must be finite.
 *   - E8M0 scale tensors of R rows and K channels use the ROW-BLOCK-MAJOR layout
 *     uint8 [ceil(R/32)][ceil(K/128)][32][4]: the scale of (row m, group g) is byte
 *       ((m/32) * ceil(K/128) + g/4) * 128 + (m%32) * 4 + g%4 .
 *     The 32 rows of one matrix-core tile then read the four scales of a 128-channel
 *     span as 128 contiguous bytes.  Bytes of groups >= K/32 are written as 0; bytes
 *     of rows >= R are never written (the buffer must still hold them).
 */
#ifndef OSC_H
#define OSC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    OSC_OK = 0,
    OSC_ERR_NULL = -1,        /* a required pointer is NULL */
    OSC_ERR_SHAPE = -2,       /* negative extent, K % 32 != 0, leading dimension < extent */
    OSC_ERR_TABLE = -3,       /* table entry outside [-1, G) or repeated inside a group */
    OSC_ERR_UNSUPPORTED = -4, /* unknown enum value, misaligned pointer or stride */
    OSC_ERR_WORKSPACE = -5,   /* a caller-provided workspace is too small */
    OSC_ERR_HIP = -6          /* the HIP runtime refused a launch */
};

enum { OSC_DT_F32 = 0, OSC_DT_BF16 = 1 };                   /* dtype of Y */
enum { OSC_FMT_MXFP4_OSC = 0, OSC_FMT_FP8_E4M3_TOKEN = 1, OSC_FMT_MXFP8 = 2,
       OSC_FMT_MXFP4_OSC_G64 = 3 };                          /* activation quantiser format */

enum { OSC_FMT16_E8M0 = 0, OSC_FMT16_NVFP4 = 1 };             /* 4-bit formats with one scale per 16 channels */

const char *osc_last_error(void);
int osc_version(void);

/* ---- offline helpers ------------------------------------------------------ */

/*
 * Suppression table -> flat channel list.  (Section 3.1: each table entry is a
 * local index in [0, G-1] naming the protected channel of its group, or -1 to
 * bypass suppression for that group.)  Generalised to R slots per group.
 *   table  host, int16 [Kg, R] row-major
 *   oidx   host, int32, room for Kg*min(R,32) entries: receives the protected
 *          global channel ids (32*g + local index) in ascending order
 *   K_o    host, receives the number of entries written
 * Errors: OSC_ERR_NULL, OSC_ERR_SHAPE (Kg < 0, R < 0), OSC_ERR_TABLE.
 */
int osc_table_to_index(const int16_t *table, int32_t Kg, int32_t R, int32_t *oidx, int32_t *K_o);

/*
 * The same conversion for the other group sizes of Section 3.1 ("Quantifying Clustering
 * Density": the channels are cut into groups of G in {16, 32, 64}; Table 2 has one row per
 * G): table entries are local indices in [0, G), group g covers channels g*G .. g*G+G-1.
 * G = 32 is osc_table_to_index.  The list it writes is what every quantiser and
 * osc_pack_weight* take, whatever G was: with G = 16 or 64 and the standard MXFP4 scale
 * block of 32 this is a protection group narrower or wider than the scale block; for scale
 * groups of 64 see OSC_FMT_MXFP4_OSC_G64 and osc_pack_weight_g.
 *   oidx   room for Kg * min(R, G) entries
 * Errors: as osc_table_to_index; OSC_ERR_UNSUPPORTED for any other G.
 */
int osc_table_to_index_g(const int16_t *table, int32_t Kg, int32_t R, int32_t G, int32_t *oidx,
                         int32_t *K_o);

/*
 * Offline weight preparation (Section 3.3.2, "zero-overhead offline weight
 * quantisation": W pre-quantised to FP4 at full shape; the weight rows of the
 * protected channels pre-stored in high precision).
 *   W      bf16 [N, ldw], unquantised weight, K % 32 == 0, ldw >= K
 *   oidx   int32 [K_o] ascending protected channel ids (device; may be NULL iff K_o == 0)
 *   Wpack  osc_packed_weight_bytes(N, K, K_o) bytes, 256-byte aligned; receives the
 *          MXFP4 codes and E8M0 scales of every row of W (nothing zeroed) and
 *          W_L[o][n] = W[n][oidx[o]] in the layout the GEMM kernels read, followed by
 *          256 bytes of zeros (what the kernels read in place of anything past the
 *          end of an operand row).  Opaque: use osc_unpack_weight to look inside.
 * osc_unpack_weight writes the plain forms back out: Wq uint8 [N, K/2]
 * (channel 2i in bits 3:0 of byte i, 2i+1 in bits 7:4), Ws uint8 [N, K/32]
 * (E8M0, plain row-major), WL bf16 [K_o, N]; any of the three may be NULL to skip it.
 */
size_t osc_packed_weight_bytes(int64_t N, int64_t K, int32_t K_o);
int osc_pack_weight(const void *W, int64_t N, int64_t K, int64_t ldw, const int32_t *oidx,
                    int32_t K_o, void *Wpack, void *stream);
int osc_unpack_weight(const void *Wpack, int64_t N, int64_t K, int32_t K_o, uint8_t *Wq,
                      uint8_t *Ws, void *WL, void *stream);

/*
 * osc_pack_weight with scale groups of G = 64 channels along K (Table 2's G = 64 row; G = 32
 * is osc_pack_weight): one shared exponent floor(log2(amax over the 64 channels)) - 2 per
 * group, stored as the code of both 32-channel blocks the group covers.  Size, layout and
 * every consumer (osc_dual_gemm, osc_grouped_dual_gemm, osc_unpack_weight) are those of
 * osc_pack_weight: the matrix core scales blocks of 32, and two equal block scales are a
 * group of 64.  K % 64 == 0.  Errors: as osc_pack_weight; OSC_ERR_UNSUPPORTED for any other G.
 */
int osc_pack_weight_g(const void *W, int64_t N, int64_t K, int64_t ldw, const int32_t *oidx,
                      int32_t K_o, int32_t G, void *Wpack, void *stream);

/*
 * FP8 fallback weights (Section 3.4): e4m3 codes with one fp32 scale per output
 * channel, scale = amax/448 (1 for rows with amax < 2^-100).
 *   W8pack  osc_packed_weight_fp8_bytes(N, K) bytes, 256-byte aligned
 * osc_unpack_weight_fp8 writes W8 uint8 [N, K] and ws float [N] (either may be NULL).
 */
size_t osc_packed_weight_fp8_bytes(int64_t N, int64_t K);
int osc_pack_weight_fp8(const void *W, int64_t N, int64_t K, int64_t ldw, void *W8pack,
                        void *stream);
int osc_unpack_weight_fp8(const void *W8pack, int64_t N, int64_t K, uint8_t *W8, float *ws,
                          void *stream);

/* ---- the hot path ----------------------------------------------------------- */

/*
 * Online activation quantiser.
 *
 * fmt = OSC_FMT_MXFP4_OSC: the OSC-enhanced quantisation workflow (Section 3.2,
 * steps 2-4; Alg. 2).  For every protected channel c = oidx[o]:
 * B[m, o] = X[m, c] (bit copy) and X[m, c] counts as +0 from then on; every
 * 32-channel group of the modified row gets an E8M0 scale with exponent
 * floor(log2(amax)) - 2 (code 0 when amax is zero or below 2^-124) and E2M1
 * elements rounded to nearest, ties to even, saturating at +-6; an element's sign
 * bit is kept even when it rounds to zero.
 *   X     bf16 [M, ldx], ldx >= K, K % 32 == 0, K <= 65536, 16-byte aligned rows (ldx % 8 == 0)
 *   oidx  int32 [K_o], ascending, distinct, each in [0, K) (as osc_table_to_index writes
 *         it; the contents are not checked on the device); NULL iff K_o == 0
 *   Xq    uint8 [M, K/2]   channel 2i -> bits 3:0 of byte i, 2i+1 -> bits 7:4
 *   Xs    E8M0 codes, row-block-major, osc_act_scale_bytes(M, K) bytes, 4-byte aligned
 *   B     bf16 [M, ldb], ldb >= K_o, ldb % 8 == 0; columns K_o..ldb-1 are set to +0.
 *         May be NULL iff K_o == 0 (then ldb is ignored).
 *
 * fmt = OSC_FMT_FP8_E4M3_TOKEN: the FP8 fallback for W_2 inputs (Section 3.4),
 * one scale per token.  amax = max_k |X[m,k]|; rows with amax < 2^-100 use
 * scale = 1; otherwise scale = amax/448 and Xq[m,k] = e4m3(X[m,k] * (448/amax)),
 * every operation one IEEE single-precision operation, e4m3 rounding to nearest
 * even.  oidx, K_o, B, ldb are ignored; K need not be a multiple of 32 but
 * must be a multiple of 8, and K <= 32768 (a row is held in registers between the
 * two phases; larger K: OSC_ERR_UNSUPPORTED).
 *   Xq    uint8 [M, K] e4m3 codes;  Xs  float [M] scales
 *
 * fmt = OSC_FMT_MXFP4_OSC_G64: OSC_FMT_MXFP4_OSC with scale groups of 64 channels (Section
 * 3.1: G in {16, 32, 64}; Table 2, row G = 64): after the protected channels are zeroed,
 * every 64 channels share one exponent floor(log2(amax)) - 2, written as the code of both
 * of their 32-channel blocks; elements, layouts, buffers and the B gather are unchanged, so
 * the result feeds osc_dual_gemm as it is.  K % 64 == 0.  The table normally names one
 * channel per 64 (osc_table_to_index_g with G = 64), but any ascending list is accepted.
 *
 * fmt = OSC_FMT_MXFP8: the 8-bit micro-scaling form of the same fallback (Section 3.4
 * allows an 8-bit micro-scaling format in place of FP8; Section 4.1, implementation
 * details: MXFP8 for the W_2 inputs).  Every 32-channel group gets an E8M0 scale with
 * exponent floor(log2(amax)) - 8 (code 0 when amax is zero or below 2^-118) and E4M3
 * elements X / 2^exponent rounded to nearest even, saturating at +-448, sign kept.
 * oidx, K_o, B, ldb are ignored; K % 32 == 0.
 *   Xq    uint8 [M, K] e4m3 codes, 8-byte aligned
 *   Xs    E8M0 codes, row-block-major, osc_act_scale_bytes(M, K) bytes, 4-byte aligned
 *
 * Errors: OSC_ERR_NULL, OSC_ERR_SHAPE, OSC_ERR_UNSUPPORTED (fmt, alignment), OSC_ERR_HIP.
 */
int osc_quantize_act(const void *X, int64_t M, int64_t K, int64_t ldx, const int32_t *oidx,
                     int32_t K_o, int fmt, uint8_t *Xq, void *Xs, void *B, int64_t ldb,
                     void *stream);

/*
 * Size in bytes of the row-block-major scale tensor of an [M, K] activation, and its
 * conversion to plain row-major uint8 [M, K/32] (for inspection and tests).
 */
size_t osc_act_scale_bytes(int64_t M, int64_t K);
int osc_unpack_act_scales(const uint8_t *Xs, int64_t M, int64_t K, uint8_t *out, void *stream);

/*
 * Dual-path GEMM (Section 3.3.1, Eq. dual-path):
 *   Y[m,n] = sum_g 2^(Xs[m,g] + Ws[n,g] - 254) * sum_{j<32} e2m1(Xq[m,32g+j]) * e2m1(Wq[n,32g+j])
 *          + sum_{o<K_o} B[m,o] * W_L[o,n]
 * (Xs[m,g] meaning the scale of row m, group g, wherever the layout puts it.)  Path A on the block-scaled FP4 matrix cores, Path B on the bf16 matrix cores,
 * both into one fp32 accumulator; Y is that accumulator, converted (round to
 * nearest even) when y_dtype is OSC_DT_BF16.
 *   Xq, Xs, B, ldb   as written by osc_quantize_act(fmt = MXFP4_OSC) with the same K, K_o
 *   Wpack            from osc_pack_weight with the same N, K, K_o
 *   Y                [M, ldy] of y_dtype, ldy >= N
 * Limits: every operand (Xq, Xs, B, one packed weight) must be smaller than 4 GiB
 * (OSC_ERR_UNSUPPORTED otherwise).  Results do not depend on which kernel the library
 * picks for a shape and are identical from run to run.
 * Errors: OSC_ERR_NULL, OSC_ERR_SHAPE, OSC_ERR_UNSUPPORTED (y_dtype, ldb % 8, size), OSC_ERR_HIP.
 */
int osc_dual_gemm(const uint8_t *Xq, const uint8_t *Xs, const void *B, int64_t ldb,
                  const void *Wpack, int64_t M, int64_t N, int64_t K, int32_t K_o, void *Y,
                  int y_dtype, int64_t ldy, void *stream);

/*
 * FP8 W8A8 GEMM (Section 3.4; also the W8A8 comparison baseline of Table 2):
 *   Y[m,n] = xs[m] * ws[n] * sum_k e4m3(X8[m,k]) * e4m3(W8[n,k])
 *   X8 uint8 [M, K], xs float [M]   from osc_quantize_act(fmt = FP8_E4M3_TOKEN)
 *   W8pack                           from osc_pack_weight_fp8; for the grouped form,
 *                                    E packs osc_packed_weight_fp8_bytes(N, K) apart
 *   expert_offsets  NULL: one problem of M rows.  Otherwise int32 [E+1] (device),
 *                   non-decreasing, expert_offsets[0] == 0, expert_offsets[E] == M:
 *                   rows [off[e], off[e+1]) use the e-th pack.
 *   K % 16 == 0.
 */
int osc_fp8_gemm(const uint8_t *X8, const float *xs, const void *W8pack, int64_t M, int64_t N,
                 int64_t K, const int32_t *expert_offsets, int32_t E, void *Y, int y_dtype,
                 int64_t ldy, void *stream);

/*
 * MXFP8 weights and GEMM (Section 3.4 / Section 4.1: the W_2 layers in MXFP8):
 *   Y[m,n] = sum_g 2^(Xs[m,g] + Ws[n,g] - 254) * sum_{j<32} e4m3(X8[m,32g+j]) * e4m3(W8[n,32g+j])
 * osc_pack_weight_mxfp8 quantises W bf16 [N, ldw] row by row as osc_quantize_act(fmt = MXFP8)
 * does and lays codes and scales out for the kernels (Wpack: osc_packed_weight_mxfp8_bytes(N, K)
 * bytes, 256-byte aligned); osc_unpack_weight_mxfp8 writes W8 uint8 [N, K] and Ws uint8
 * [N, K/32] (plain row-major), either may be NULL.
 *   X8, Xs          from osc_quantize_act(fmt = MXFP8) with the same K
 *   expert_offsets  as in osc_fp8_gemm (E packs osc_packed_weight_mxfp8_bytes(N, K) apart)
 *   K % 128 == 0 (OSC_ERR_UNSUPPORTED otherwise: only whole 128-channel lines are implemented)
 */
size_t osc_packed_weight_mxfp8_bytes(int64_t N, int64_t K);
int osc_pack_weight_mxfp8(const void *W, int64_t N, int64_t K, int64_t ldw, void *Wpack, void *stream);
int osc_unpack_weight_mxfp8(const void *Wpack, int64_t N, int64_t K, uint8_t *W8, uint8_t *Ws,
                            void *stream);
int osc_mxfp8_gemm(const uint8_t *X8, const uint8_t *Xs, const void *Wpack, int64_t M, int64_t N,
                   int64_t K, const int32_t *expert_offsets, int32_t E, void *Y, int y_dtype,
                   int64_t ldy, void *stream);

/*
 * Grouped dual-path GEMM for mixture-of-experts layers (the MoE model of
 * Section 4.1): the dual-path GEMM above for E independent experts that share
 * K, N and the suppression table.
 *   T               number of routed rows (sum of the experts' row counts)
 *   expert_offsets  int32 [E+1] (device), non-decreasing, [0] == 0, [E] == T
 *   row_map         int32 [T] (device) or NULL: routed row t reads row row_map[t]
 *                   of Xq/Xs/B (NULL: row t).  Y row t is written for every t.
 *   Wpack           E packs, osc_packed_weight_bytes(N, K, K_o) bytes apart
 */
int osc_grouped_dual_gemm(const uint8_t *Xq, const uint8_t *Xs, const void *B, int64_t ldb,
                          const int32_t *row_map, const int32_t *expert_offsets, int32_t E,
                          int64_t T, const void *Wpack, int64_t N, int64_t K, int32_t K_o,
                          void *Y, int y_dtype, int64_t ldy, void *stream);

/*
 * RMSNorm fused with the OSC-enhanced quantiser: what osc_quantize_act(fmt = OSC_FMT_MXFP4_OSC)
 * returns for the normalised row y = x / sqrt(mean(x^2) + eps) * gamma, without y passing
 * through memory (the inputs of the attention and FFN projections, positions 1 and 3 of
 * Section 2.1, are RMSNorm outputs).  The normalisation is defined so that its result does not
 * depend on any order of summation:
 *   e    = the largest biased bf16 exponent field of the row (at least 1);
 *   S    = sum over the row of floor(m^2 * 2^28 / 4^(e - E)), |x| = m * 2^(E - 134), m an 8-bit
 *          integer, E >= 1 (64-bit integer; terms 2^44 below the largest vanish);
 *   r    = (float)(1 / sqrt((double)S * 2^(2e - 296) / K + eps)), double arithmetic;
 *   y    = bf16(bf16(x * r) * gamma), single-precision products, round to nearest even.
 *   gamma  bf16 [K] (device), 16-byte aligned;  eps >= 0
 *   Xn     bf16 [M, K] (device) or NULL: receives y when given
 *   K <= 12288; everything else as osc_quantize_act.
 */
int osc_rmsnorm_quantize_act(const void *X, const void *gamma, float eps, int64_t M, int64_t K,
                             int64_t ldx, const int32_t *oidx, int32_t K_o, uint8_t *Xq, void *Xs,
                             void *B, int64_t ldb, void *Xn, void *stream);

/*
 * SwiGLU fused with the MXFP8 quantiser of the W_2 fallback (the W_2 inputs, position 4 of
 * Section 2.1, are silu(gate) * up; Section 4.1 quantises them to MXFP8): what
 * osc_quantize_act(fmt = OSC_FMT_MXFP8) returns for y = bf16(bf16(silu(g)) * u), without y
 * passing through memory.  silu(g) = g / (1 + exp(-g)) is computed as a fixed sequence of
 * correctly rounded single-precision operations: z = clamp(-g, -86, 86); n = rint(z * log2 e);
 * r = fma(n, -LN2_HI, z), r = fma(n, -LN2_LO, r) with LN2_HI = 0x1.62e4p-1, LN2_LO =
 * 0x1.7f7d1cp-20; p = Horner of 1 + r + r^2/2 + ... + r^6/720, one fma per step from the
 * highest term; e = p * 2^n; silu = g / (1 + e).
 *   G, U  bf16 [M, ldg], [M, ldu] (device), 16-byte aligned rows: gate and up projections (two
 *         halves of one fused GEMM output are fine: pass the pointers and the common stride)
 *   Xq    uint8 [M, K] E4M3 codes; Xs E8M0 scales as for OSC_FMT_MXFP8
 *   Yn    bf16 [M, K] (device) or NULL: receives y when given
 * From a few million elements on, this call and osc_swiglu_quantize_act_fp8 first tabulate
 * bf16(silu(g)) for all 65536 bf16 values of g with the arithmetic above (a second small kernel on
 * the same stream, into 128 KB of device memory that the library owns) and look the values up;
 * the results are the same bits.  Calls that overlap on one device rewrite the table with
 * identical contents.
 * Errors as osc_quantize_act.
 */
int osc_swiglu_quantize_act(const void *G, const void *U, int64_t M, int64_t K, int64_t ldg,
                            int64_t ldu, uint8_t *Xq, void *Xs, void *Yn, void *stream);

/*
 * The same producer fused with the per-token FP8 quantiser (Section 3.4, the e4m3 form of the
 * W_2 fallback that osc_fp8_gemm multiplies): what osc_quantize_act(fmt =
 * OSC_FMT_FP8_E4M3_TOKEN) returns for y = bf16(bf16(silu(g)) * u), silu as defined above.
 *   G, U  as above; K % 8 == 0, K <= 16384
 *   X8    uint8 [M, K] e4m3 codes;  xs  float [M] scales (amax/448, or 1 for rows below 2^-100)
 *   Yn    bf16 [M, K] (device) or NULL: receives y when given
 * Errors as osc_quantize_act.
 */
int osc_swiglu_quantize_act_fp8(const void *G, const void *U, int64_t M, int64_t K, int64_t ldg,
                                int64_t ldu, uint8_t *X8, float *xs, void *Yn, void *stream);

/*
 * "Dynamic" protection, the control experiment of Section 4.2 (Table 3, note 3: per-group
 * maximum value detection at run time).  Like osc_quantize_act(fmt = OSC_FMT_MXFP4_OSC) with
 * one slot per group, except that the protected position is chosen per token: the largest
 * magnitude of the group (the lowest position among equal magnitudes).
 *   Bd   bf16 [M, ldb], ldb >= K, ldb % 8 == 0, 16-byte aligned: the backed-up values in
 *        place (Bd[m, c] = X[m, c] for the protected channel of each group, +0 elsewhere).
 *        With weights packed for all K channels (oidx = 0..K-1) it is the B operand of
 *        osc_dual_gemm: on hardware without per-token gathers the scheme costs a full
 *        bf16 branch, which is the overhead the static table removes.
 *   idx  uint8 [M, K/32] or NULL: the chosen local positions (4-byte aligned)
 *   Xq, Xs as for OSC_FMT_MXFP4_OSC.
 * Errors as osc_quantize_act.
 */
int osc_quantize_act_dynamic(const void *X, int64_t M, int64_t K, int64_t ldx, uint8_t *Xq,
                             void *Xs, void *Bd, int64_t ldb, uint8_t *idx, void *stream);

/* ---- 4-bit formats with one scale per 16 channels --------------------------------------------- */

/*
 * The OSC quantiser and the dual-path layer for the 4-bit formats whose scale group is 16 channels
 * (Section 3.1: group sizes G in {16, 32, 64}, chosen to line up with the scale groups of
 * micro-scaling formats; Table 2, row G = 16; the abstract and the conclusion name NVFP4).  The paper gives no
 * arithmetic for either; this library reads them as follows.
 *   OSC_FMT16_E8M0   E2M1 elements, one E8M0 scale per 16 channels with exponent floor(log2 amax) - 2
 *                    (code 0 for amax zero or below 2^-124); elements X / 2^exponent, nearest even,
 *                    saturating at +-6.  The tensor scale arguments are ignored.
 *   OSC_FMT16_NVFP4  E2M1 elements, one E4M3 scale per 16 channels, one single-precision scale ts per
 *                    tensor, supplied by the caller (a calibrated constant, typically the largest
 *                    magnitude of the tensor divided by 6 * 448; 2^-100 <= ts <= 2^100).  Every step
 *                    is one IEEE single-precision operation: d = 6 * ts; q = amax / d; scale byte =
 *                    e4m3(q), nearest even, saturating at 448; s = value of the byte; inv = 1 / (ts * s)
 *                    (0 when s is 0); element = e2m1(x * inv), nearest even, saturating.
 * In both, Alg. 2 is unchanged: B[m, o] = X[m, oidx[o]] and those channels count as +0 before their
 * block's scale is computed; an element keeps its sign bit when it rounds to zero.
 *
 * osc_quantize_act_g16:  X, oidx, K_o, B, ldb as in osc_quantize_act; K % 64 == 0;
 *   Xq    uint8 [M, K/2], channel 2i in bits 3:0 of byte i;  Xs16  uint8 [M, K/16], plain row-major.
 * osc_pack_weight_g16:  quantises W bf16 [N, ldw] row by row in the same format (nothing zeroed),
 *   gathers W_L[o][n] = W[n][oidx[o]]; Wpack: osc_packed_weight_g16_bytes(N, K, K_o) bytes, 256-byte
 *   aligned, opaque (osc_unpack_weight_g16 writes Wq uint8 [N, K/2], Ws16 uint8 [N, K/16], WL bf16
 *   [K_o, N]; any may be NULL).
 * osc_dual_gemm_g16:
 *   Y[m,n] = xts * wts * sum_b s(Xs16[m,b]) * s(Ws16[n,b]) * sum_{j<16} e2m1(Xq[m,16b+j]) * e2m1(Wq[n,16b+j])
 *          + sum_{o<K_o} B[m,o] * W_L[o,n]          (xts = wts = 1 for OSC_FMT16_E8M0)
 *   K % 256 == 0; ldb % 64 == 0.  The matrix core multiplies 4-bit operands only with one power-of-two
 *   scale per 32 channels, so this kernel expands the codes to bf16 in registers (exactly) and uses the
 *   bf16 matrix core: it is built for the weight-bound regime (a few tokens, Table 2's left column),
 *   where the formats' gain is the 0.56 bytes per weight that travel; it accepts any M, at the bf16
 *   matrix rate.
 * Errors: OSC_ERR_NULL, OSC_ERR_SHAPE, OSC_ERR_UNSUPPORTED (format, alignment, K), OSC_ERR_HIP.
 */
int osc_quantize_act_g16(const void *X, int64_t M, int64_t K, int64_t ldx, const int32_t *oidx,
                         int32_t K_o, int fmt16, float tensor_scale, uint8_t *Xq, uint8_t *Xs16,
                         void *B, int64_t ldb, void *stream);
size_t osc_packed_weight_g16_bytes(int64_t N, int64_t K, int32_t K_o);
int osc_pack_weight_g16(const void *W, int64_t N, int64_t K, int64_t ldw, const int32_t *oidx,
                        int32_t K_o, int fmt16, float tensor_scale, void *Wpack, void *stream);
int osc_unpack_weight_g16(const void *Wpack, int64_t N, int64_t K, int32_t K_o, uint8_t *Wq,
                          uint8_t *Ws16, void *WL, void *stream);
int osc_dual_gemm_g16(const uint8_t *Xq, const uint8_t *Xs16, float x_tensor_scale, const void *B,
                      int64_t ldb, const void *Wpack, float w_tensor_scale, int64_t M, int64_t N,
                      int64_t K, int32_t K_o, int fmt16, void *Y, int y_dtype, int64_t ldy,
                      void *stream);

/* ---- offline profiling (calibration) ------------------------------------------ */

/*
 * Layer-wise outlier threshold (Section 2.1, Eq. 1): T = alpha * mean |x| over all
 * tokens and channels of one activation interface (alpha = 5 in the paper).
 * Two calls, so that a calibration set can be fed in pieces:
 *   osc_profile_abs_sum    *abs_sum += sum of |x| over X.  The caller zeroes *abs_sum
 *                          before the first piece.  Added with floating-point atomics:
 *                          the order of the additions, and so the last bits of the
 *                          double, can differ from run to run.
 *   osc_profile_threshold  *T = (float)(alpha * *abs_sum / count), count = the number
 *                          of elements summed (tokens x channels over all pieces)
 *   X        bf16 [S, ldx] (device), ldx >= H, H % 8 == 0, rows 16-byte aligned; finite values
 *   abs_sum  double (device), T float (device)
 * Errors: OSC_ERR_NULL, OSC_ERR_SHAPE, OSC_ERR_UNSUPPORTED (alignment), OSC_ERR_HIP.
 */
int osc_profile_abs_sum(const void *X, int64_t S, int64_t H, int64_t ldx, double *abs_sum,
                        void *stream);
int osc_profile_threshold(const double *abs_sum, int64_t count, float alpha, float *T,
                          void *stream);

/*
 * Candidate sets of Alg. 1 as counts (Section 2.2, Eq. 2 and Eq. 3).  For every token s
 * and every group k of G consecutive channels: j* = the local index of the largest
 * magnitude in the group (the lowest index among equal magnitudes); when that magnitude
 * is strictly above *T, hist[k*G + j*] grows by one.  Counts are added to what hist
 * holds (zero it before the first piece); integer atomics, so the result is exact and
 * independent of any ordering.
 *   G     16, 32 or 64 (the group sizes of Section 2.2); H % G == 0
 *   T     float (device): the threshold; a negative value admits every token, NaN none
 *   hist  uint32 [H/G, G] (device) -- one counter per channel
 */
int osc_profile_hist(const void *X, int64_t S, int64_t H, int64_t ldx, int32_t G, const float *T,
                     uint32_t *hist, void *stream);

/*
 * Suppression table entries and clustering density from the counts (Alg. 1; Section 2.2,
 * Eq. 4 and the definition of the density after it).
 *   table    int16 [Kg, R] (device): the R local indices with the largest counts, most
 *            frequent first, the lower index first among equal counts; only indices
 *            whose count is above zero, -1 otherwise.  Column 0 is the table of Alg. 1
 *            (the mode of the candidate set, -1 when the set is empty).  Copied to the
 *            host it is what osc_table_to_index takes (for G = 32).
 *   n_total  uint32 [Kg] or NULL: tokens in the group's candidate set (N_total)
 *   n_hit    uint32 [Kg] or NULL: the largest count (N_hit)
 *   density  float [Kg] or NULL: C_k = N_hit / N_total, 0 for an empty set
 *   cbar     float or NULL: mean of C_k over the groups whose set is not empty (0 if none)
 *   G in [1, 64].  All pointers are device pointers.
 */
int osc_profile_table(const uint32_t *hist, int32_t Kg, int32_t G, int32_t R, int16_t *table,
                      uint32_t *n_total, uint32_t *n_hit, float *density, float *cbar,
                      void *stream);

/*
 * Alg. 1 for one activation interface in one call: Eq. 1's threshold over X, the candidate counts
 * of Eq. 2-3, and the table, densities and mean density of Eq. 4, i.e. osc_profile_abs_sum,
 * osc_profile_threshold, osc_profile_hist and osc_profile_table in sequence on one calibration
 * piece X[S, H] (S > 0, H > 0).  The intermediate results live in `workspace`.
 *   T_out            float (device) or NULL: receives the threshold that was used
 *   workspace        device memory, 256-byte aligned, osc_profile_workspace_bytes(H) bytes
 *                    (= 256 + 4*H); cleared by the call itself, contents afterwards unspecified
 *   everything else as in the four calls above (table int16 [H/G, R], ...).
 * Errors: those of the four calls; OSC_ERR_WORKSPACE when workspace_bytes is too small.
 */
size_t osc_profile_workspace_bytes(int64_t H);
int osc_profile_calibrate(const void *X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha,
                          int32_t R, int16_t *table, uint32_t *n_total, uint32_t *n_hit,
                          float *density, float *cbar, float *T_out, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * osc_profile_calibrate for callers that cannot allocate device memory or have none to spare for a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments without the workspace, same results.  The intermediate results live in a fixed
 * 64.25 KB array inside the library (one copy on every GPU the library runs on, kept until the
 * process ends), so H <= 16384 (OSC_ERR_UNSUPPORTED above that).  The call allocates nothing and
 * clears the part of the array it uses itself.  Every call on one GPU uses that GPU's one array:
 * calls that overlap on the same GPU (different streams, different threads) race and give wrong
 * results; calls on one stream, or otherwise ordered, are fine.
 */
int osc_profile_calibrate_static(const void *X, int64_t S, int64_t H, int64_t ldx, int32_t G,
                                 float alpha, int32_t R, int16_t *table, uint32_t *n_total,
                                 uint32_t *n_hit, float *density, float *cbar, float *T_out,
                                 void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OSC_H */
