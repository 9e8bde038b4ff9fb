/*
 * CPU oracle for the OSC dual-path linear layer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain reference that the HIP kernels are checked
 * against.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may link or call it; the product library never does and
 * shares no source, header, table or constant generator with it.
 *
 * What it computes, and the passage of the paper each function follows:
 *   ref_table_to_index      suppression vector I = L[p][l] (Section 3.1, Alg. 1
 *                           output form: one local index per group or -1)
 *   ref_quantize_mxfp4_osc  OSC-enhanced quantisation (Section 3.2 steps 1-4,
 *                           Alg. 2): extract to buffer B, zero, micro-scale
 *                           quantise.  "Standard micro-scaling" is read as
 *                           OCP MX v1.0 MXFP4: one E8M0 scale per 32 elements,
 *                           shared exponent floor(log2 amax) - 2, E2M1 elements
 *                           rounded to nearest, ties to even, saturating.
 *   ref_quantize_mxfp4_dynamic  the "Dynamic" protection control of Section 4.2 (Table 3,
 *                           note 3): the protected element of a group is found
 *                           at run time, per token, as the group's largest
 *                           magnitude; everything else as in Alg. 2
 *   ref_rmsnorm             the normalisation that produces the inputs of the attention
 *                           and FFN projections (positions 1 and 3 of Section 2.1,
 *                           Figure 1), in a form whose result does not depend on
 *                           the order of any summation, so that a producer fused
 *                           with the quantiser can be compared bit for bit
 *   ref_swiglu              the gated activation that produces the W_2 inputs (position 4 of
 *                           Section 2.1), y = silu(gate) * up, as a fixed sequence of
 *                           correctly rounded single-precision operations, so that a producer
 *                           fused with the 8-bit quantiser can be compared bit for bit
 *   ref_rmsnorm_plain, ref_swiglu_plain  the same two producers in plain double precision with a
 *                           single final rounding: the pin that ties the two recipes above (and the
 *                           kernels that reproduce them) to RMSNorm and SwiGLU themselves
 *   ref_quantize_fp4_g16, ref_dual_gemm_g16  Alg. 2 and Eq. (dual-path) for 4-bit formats whose scale
 *                           group is 16 channels (Section 3.1's G = 16; Table 2's first row; the
 *                           NVFP4 format named in the abstract and the conclusion)
 *   ref_gather_wl           W_L: rows of the high-precision weight named by
 *                           the same table (Section 3.3.1, second bullet)
 *   ref_dual_gemm           Eq. (dual-path): Y = (Q_X (x) Q_W).S + B.W_L
 *   ref_quantize_fp8_rows   FP8 fallback quantiser (Section 3.4), read as
 *                           e4m3 with one fp32 scale per row (per token for
 *                           activations, per output channel for weights)
 *   ref_fp8_gemm            the W8A8 linear layer on those operands
 *   ref_grouped_*           the same two GEMMs for E independent experts
 *                           (MoE model of Section 4.1)
 *   ref_quantize_mxfp8      the 8-bit micro-scaling form of the fallback
 *                           (Section 3.4 allows an 8-bit micro-scaling format
 *                           there; Section 4.1 implementation details:
 *                           MXFP8 for the W_2 inputs), read as OCP MX v1.0
 *                           MXFP8 with E4M3 elements: one E8M0 scale per 32
 *                           elements, shared exponent floor(log2 amax) - 8,
 *                           elements rounded to nearest even, saturating
 *   ref_mxfp8_gemm          the linear layer on two MXFP8 operands
 *   ref_profile_threshold   layer-wise outlier threshold T_l = alpha * mean|X| (Eq. 1)
 *   ref_profile_hist        per group and local index: number of tokens whose
 *                           largest-magnitude element of the group sits at that
 *                           index and exceeds T_l (Eq. 2, Eq. 3; the candidate
 *                           sets of Alg. 1 kept as counts)
 *   ref_profile_table       suppression table entry = mode of the candidate set,
 *                           -1 when it is empty (Alg. 1); N_total, N_hit,
 *                           clustering density C_k and its mean (Eq. 4 and the
 *                           paragraph after it); extended to the R most frequent
 *                           indices per group
 *
 * Floating point: every GEMM accumulates in double.  The FP8 quantiser's
 * scale arithmetic is IEEE single precision (one division, one multiply),
 * because it decides integer codes and both sides must take that decision
 * in the same precision.
 *
 * Parity pins: tests/test_oracle_*.py.  Non-finite inputs are outside the
 * contract: every quantiser returns REF_ERR_NONFINITE when it meets one.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC osc_ref.c -lm
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_ERR_ARG (-1)
#define REF_ERR_TABLE (-3)
#define REF_ERR_NONFINITE (-7)

#define G 32 /* MXFP4 block size (Section 4.1, implementation details) */

/* ---- number formats ---------------------------------------------------- */

static float bf16_to_float(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* E2M1 magnitudes by 3-bit code {exp[1:0], man}; bit 3 of a code is the sign. */
static const double E2M1_MAG[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

double ref_e2m1_decode(int code) {
    double m = E2M1_MAG[code & 7];
    return (code & 8) ? -m : m;
}

/* Nearest E2M1 magnitude to |v|; a value half-way between two neighbours goes
 * to the one whose mantissa bit (code bit 0) is 0; anything above the largest
 * magnitude saturates to it (stated first, so that the distance comparison
 * below never sees a magnitude large enough to absorb the grid values). */
static int e2m1_nearest_mag_code(double a) {
    if (a > E2M1_MAG[7]) return 7;
    int best = 0;
    double bd = fabs(a - E2M1_MAG[0]);
    for (int c = 1; c < 8; ++c) {
        double d = fabs(a - E2M1_MAG[c]);
        if (d < bd || (d == bd && (c & 1) == 0)) {
            best = c;
            bd = d;
        }
    }
    return best;
}

/* Shared exponent of one MX block: floor(log2(amax)) - emax of the element
 * format (2 for E2M1, 8 for E4M3), clamped to the E8M0 range [-127, 127];
 * amax == 0 takes the lower clamp. */
static int mx_shared_exponent_for(double amax, int emax_elem) {
    if (amax == 0.0) return -127;
    int ex;
    (void)frexp(amax, &ex); /* amax = m * 2^ex, m in [0.5, 1) */
    int e = (ex - 1) - emax_elem;
    if (e < -127) e = -127;
    if (e > 127) e = 127;
    return e;
}
static int mx_shared_exponent(double amax) { return mx_shared_exponent_for(amax, 2); }

int ref_e8m0_code_for_amax(double amax) { return mx_shared_exponent(amax) + 127; }
int ref_e8m0_code_for_amax_e4m3(double amax) { return mx_shared_exponent_for(amax, 8) + 127; }

int ref_e2m1_encode(double v, int negative) {
    return e2m1_nearest_mag_code(fabs(v)) | (negative ? 8 : 0);
}

/* OCP E4M3: bias 7, 3 mantissa bits, no infinity, largest finite 448,
 * subnormal step 2^-9. */
double ref_e4m3_decode(int code) {
    int s = (code >> 7) & 1, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        v = ldexp((double)m, -9);
    else
        v = ldexp(1.0 + m / 8.0, e - 7);
    return s ? -v : v;
}

/* Round a finite float to E4M3, nearest-even, saturating at +-448.
 * The quantum of the binade holding |v| is 2^(floor(log2|v|) - 3), never
 * below the subnormal step 2^-9; rint() rounds half to even. */
int ref_e4m3_encode(float vf) {
    double v = (double)vf;
    int sign = signbit(v) ? 0x80 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (!(a <= DBL_MAX)) return sign | 0x7F; /* not finite: outside the contract (callers report an error) */
    int ex;
    (void)frexp(a, &ex);
    int p = ex - 1; /* floor(log2 a) */
    if (p < -6) p = -6;
    double q = ldexp(1.0, p - 3);
    double r = rint(a / q) * q; /* a/q is exact: q is a power of two */
    if (r > 448.0) r = 448.0;
    if (r == 0.0) return sign;
    /* encode the representable value r */
    (void)frexp(r, &ex);
    p = ex - 1;
    int e, m;
    if (p < -6) {
        e = 0;
        m = (int)ldexp(r, 9);
    } else {
        e = p + 7;
        m = (int)(ldexp(r, -p) * 8.0) - 8;
    }
    return sign | (e << 3) | m;
}

/* ---- table ------------------------------------------------------------- */

/* Paper-form table: Kg groups of Gs channels x R slots, each a local index in
 * [0, Gs) or -1 (no suppression); the paper's group sizes are 16, 32 and 64
 * (Section 3.1, "Quantifying Clustering Density").  Output: the flat list of
 * protected global channel ids in ascending order, and its length K_o. */
int ref_table_to_index_g(const int16_t *table, int32_t Kg, int32_t R, int32_t Gs, int32_t *oidx,
                         int32_t *K_o) {
    if (!table || !oidx || !K_o || Kg < 0 || R < 0 || Gs < 1 || Gs > 64) return REF_ERR_ARG;
    int32_t n = 0;
    for (int32_t g = 0; g < Kg; ++g) {
        uint64_t seen = 0;
        for (int32_t s = 0; s < R; ++s) {
            int j = table[(int64_t)g * R + s];
            if (j == -1) continue;
            if (j < 0 || j >= Gs) return REF_ERR_TABLE;
            if (seen & ((uint64_t)1 << j)) return REF_ERR_TABLE;
            seen |= (uint64_t)1 << j;
        }
        for (int j = 0; j < Gs; ++j)
            if (seen & ((uint64_t)1 << j)) oidx[n++] = g * Gs + j;
    }
    *K_o = n;
    return REF_OK;
}
int ref_table_to_index(const int16_t *table, int32_t Kg, int32_t R, int32_t *oidx, int32_t *K_o) {
    return ref_table_to_index_g(table, Kg, R, G, oidx, K_o);
}

/* ---- OSC-enhanced MXFP4 quantiser (Alg. 2) ------------------------------ */

/* X[M, K] bf16 bits, row stride ldx.  oidx[K_o]: protected channel ids.
 * Outputs: Xq[M, K/2] (element 2i in bits 3:0, 2i+1 in bits 7:4),
 * Xs[M, K/32] E8M0 codes, B[M, ldb] bf16 bits with column o = the original
 * value of channel oidx[o] and columns K_o..ldb-1 = +0.
 * Gs is the size of a scale group: 32 (the MXFP4 block) or 64 (Table 2's
 * G = 64 row: one shared exponent for 64 channels, held in the two stored
 * blocks of 32 that the group covers, so the GEMM below needs no change). */
int ref_quantize_mxfp4_osc_g(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                             const int32_t *oidx, int32_t K_o, int32_t Gs, uint8_t *Xq, uint8_t *Xs,
                             uint16_t *B, int64_t ldb) {
    if (Gs != 32 && Gs != 64) return REF_ERR_ARG;
    if (M < 0 || K < 0 || K % Gs || ldx < K || K_o < 0 || ldb < K_o) return REF_ERR_ARG;
    if (M == 0 || K == 0) return REF_OK;
    if (!X || !Xq || !Xs || (K_o && (!oidx || !B))) return REF_ERR_ARG;
    for (int32_t o = 0; o < K_o; ++o)
        if (oidx[o] < 0 || oidx[o] >= K) return REF_ERR_TABLE;
    int64_t Kg = K / G;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        /* the suppression flags of this row (the same for every row) */
        uint8_t removed[K];
        memset(removed, 0, (size_t)K);
        /* steps 2-3: back up the protected values, then zero them */
        if (B) {
            for (int64_t o = 0; o < ldb; ++o) B[m * ldb + o] = 0;
        }
        for (int32_t o = 0; o < K_o; ++o) {
            B[m * ldb + o] = x[oidx[o]];
            removed[oidx[o]] = 1;
        }
        /* step 4: scale and quantise the modified tensor, group by group */
        for (int64_t g = 0; g < K / Gs; ++g) {
            double v[64];
            int neg[64];
            double amax = 0.0;
            for (int j = 0; j < Gs; ++j) {
                uint16_t h = removed[g * Gs + j] ? (uint16_t)0 : x[g * Gs + j];
                if ((h & 0x7F80) == 0x7F80) bad = 1;
                v[j] = (double)bf16_to_float(h);
                neg[j] = (h >> 15) & 1;
                if (fabs(v[j]) > amax) amax = fabs(v[j]);
            }
            int e = mx_shared_exponent(amax);
            /* one code per stored block of 32: a group of 64 writes the same code twice */
            for (int b = 0; b < Gs / G; ++b) Xs[m * Kg + g * (Gs / G) + b] = (uint8_t)(e + 127);
            for (int j = 0; j < Gs; j += 2) {
                int lo = ref_e2m1_encode(ldexp(v[j], -e), neg[j]);
                int hi = ref_e2m1_encode(ldexp(v[j + 1], -e), neg[j + 1]);
                Xq[m * (K / 2) + (g * Gs + j) / 2] = (uint8_t)(lo | (hi << 4));
            }
        }
    }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}
int ref_quantize_mxfp4_osc(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                           const int32_t *oidx, int32_t K_o, uint8_t *Xq, uint8_t *Xs,
                           uint16_t *B, int64_t ldb) {
    return ref_quantize_mxfp4_osc_g(X, M, K, ldx, oidx, K_o, G, Xq, Xs, B, ldb);
}

/* RMSNorm, y = x / sqrt(mean(x^2) + eps) * gamma, defined so that every step is exact or a single
 * correctly rounded IEEE operation, none of which depends on an order of summation:
 *   1. e = the largest biased exponent field of the row (a subnormal counts as 1);
 *   2. every |x| = m * 2^(E - 134) with an 8-bit integer m (hidden bit included) and E >= 1; its
 *      square enters a 64-bit fixed-point sum in units of 2^(2e - 296):
 *      S = sum of floor(m^2 * 2^28 / 2^(2(e - E)))   (terms more than 2^44 below the largest vanish);
 *   3. mean = (double)S * 2^(2e - 296) / K, r = (float)(1 / sqrt(mean + eps)) in double arithmetic;
 *   4. t = bf16(x * r) with one single-precision multiplication, y = bf16(t * gamma) (that product
 *      is exact in single precision); bf16() rounds to nearest, ties to even.
 * X, Y: bf16 bits [M, K] (row strides ldx, K); gamma: bf16 bits [K]. */
static uint16_t float_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int ref_rmsnorm(const uint16_t *X, const uint16_t *gamma, double eps, int64_t M, int64_t K, int64_t ldx,
                uint16_t *Y) {
    if (M < 0 || K <= 0 || K > 65536 || ldx < K || !X || !gamma || !Y) return REF_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        int e = 1;
        for (int64_t j = 0; j < K; ++j) {
            if ((x[j] & 0x7F80) == 0x7F80) bad = 1;
            int E = (x[j] >> 7) & 0xFF;
            if (E > e) e = E;
        }
        uint64_t S = 0;
        for (int64_t j = 0; j < K; ++j) {
            int E = (x[j] >> 7) & 0xFF;
            uint64_t mant = x[j] & 0x7F;
            if (E == 0) E = 1; else mant |= 0x80;
            int sh = 2 * (e - E);
            if (sh < 64) S += ((mant * mant) << 28) >> sh;
        }
        double mean = ldexp((double)S, 2 * e - 296) / (double)K;
        float r = (float)(1.0 / sqrt(mean + eps));
        for (int64_t j = 0; j < K; ++j) {
            if ((gamma[j] & 0x7F80) == 0x7F80) bad = 1;
            float t = bf16_to_float(float_to_bf16_rne(bf16_to_float(x[j]) * r));
            Y[m * K + j] = float_to_bf16_rne(t * bf16_to_float(gamma[j]));
        }
    }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}

/* SwiGLU, y = bf16(bf16(silu(g)) * u) with silu(g) = g / (1 + exp(-g)), every step one IEEE single
 * precision operation (fmaf is the fused multiply-add, one rounding):
 *   z = min(max(-g, -86), 86)                      (keeps 2^n normal; beyond it silu is g or ~0 anyway)
 *   n = rint(z * log2(e));  r = fma(n, -LN2_HI, z);  r = fma(n, -LN2_LO, r)
 *   p = 1 + r(1 + r(1/2 + r(1/6 + r(1/24 + r(1/120 + r/720)))))   (Horner, one fma per step)
 *   e = p * 2^n (exact);  s = g / (1 + e)           (one addition, one division)
 * G, U: bf16 bits [M, K] with row strides ldg, ldu; Y: bf16 bits [M, K]. */
static float silu_f32(float g) {
    const float LOG2E = 0x1.715476p+0f, LN2_HI = 0x1.62e400p-1f, LN2_LO = 0x1.7f7d1cp-20f;
    float z = -g;
    if (z < -86.0f) z = -86.0f;
    if (z > 86.0f) z = 86.0f;
    float n = rintf(z * LOG2E);
    float r = fmaf(n, -LN2_HI, z);
    r = fmaf(n, -LN2_LO, r);
    float p = 1.0f / 720.0f;
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    float e = ldexpf(p, (int)n);
    return g / (1.0f + e);
}

int ref_swiglu(const uint16_t *Gt, const uint16_t *U, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
               uint16_t *Y) {
    if (M < 0 || K < 0 || ldg < K || ldu < K || (M && K && (!Gt || !U || !Y))) return REF_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j = 0; j < K; ++j) {
            uint16_t g = Gt[m * ldg + j], u = U[m * ldu + j];
            if ((g & 0x7F80) == 0x7F80 || (u & 0x7F80) == 0x7F80) bad = 1;
            float t = bf16_to_float(float_to_bf16_rne(silu_f32(bf16_to_float(g))));
            Y[m * K + j] = float_to_bf16_rne(t * bf16_to_float(u));
        }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}

/* The textbook forms of the two producers, written without any of the devices above: every
 * quantity in double precision (the sum of squares in plain double accumulation, sqrt and exp from
 * libm) and ONE rounding to bf16 at the very end, or, with mid_round, the two roundings that a model
 * made of bf16 modules performs (after the normalisation / after silu, then after the product).
 * They do not define the fused kernels' bits (the
 * recipes above do, and those were shaped so that a kernel can reproduce them exactly); they pin
 * the recipes, and through them the kernels, to RMSNorm and SwiGLU themselves: results may differ
 * from ref_rmsnorm / ref_swiglu by at most one bf16 step, and rarely do. */
static uint16_t double_to_bf16_rne(double v) {
    /* nearest bf16 of a finite double (ties to even), through the exact neighbours in float */
    float f = (float)v;             /* 24 significant bits: may itself sit on a bf16 tie by rounding, */
    uint32_t u;                     /* so decide by comparing v with the two bf16 neighbours exactly   */
    memcpy(&u, &f, 4);
    uint32_t lo = u & 0xFFFF0000u, hi = lo + 0x10000u;
    float flo, fhi;
    memcpy(&flo, &lo, 4);
    memcpy(&fhi, &hi, 4);
    double dlo = fabs(v - (double)flo), dhi = fabs((double)fhi - v);
    if (dlo < dhi) return (uint16_t)(lo >> 16);
    if (dhi < dlo) return (uint16_t)(hi >> 16);
    return (uint16_t)(((lo >> 16) & 1u) ? (hi >> 16) : (lo >> 16));
}

/* mid_round = 1 also rounds the normalised value (the gated value) to bf16 before the last
 * product, as a model whose modules exchange bf16 tensors does; 0 rounds once, at the end. */
int ref_rmsnorm_plain(const uint16_t *X, const uint16_t *gamma, double eps, int64_t M, int64_t K, int64_t ldx,
                      int mid_round, uint16_t *Y) {
    if (M < 0 || K <= 0 || ldx < K || !X || !gamma || !Y) return REF_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        double ss = 0.0;
        for (int64_t j = 0; j < K; ++j) {
            double v = (double)bf16_to_float(x[j]);
            ss += v * v;
        }
        double r = 1.0 / sqrt(ss / (double)K + eps);
        for (int64_t j = 0; j < K; ++j) {
            double t = (double)bf16_to_float(x[j]) * r;
            if (mid_round) t = (double)bf16_to_float(double_to_bf16_rne(t));
            Y[m * K + j] = double_to_bf16_rne(t * (double)bf16_to_float(gamma[j]));
        }
    }
    return REF_OK;
}

int ref_swiglu_plain(const uint16_t *Gt, const uint16_t *U, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                     int mid_round, uint16_t *Y) {
    if (M < 0 || K < 0 || ldg < K || ldu < K || (M && K && (!Gt || !U || !Y))) return REF_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j = 0; j < K; ++j) {
            double g = (double)bf16_to_float(Gt[m * ldg + j]), u = (double)bf16_to_float(U[m * ldu + j]);
            double t = g / (1.0 + exp(-g));
            if (mid_round) t = (double)bf16_to_float(double_to_bf16_rne(t));
            Y[m * K + j] = double_to_bf16_rne(t * u);
        }
    return REF_OK;
}

/* Dynamic protection (Section 4.2: per-group maximum value detection at run time).  For every
 * token and every group of 32 channels: j* = the position of the largest magnitude (the lowest
 * position among equal magnitudes); that element is backed up, zeroed and the rest of the group
 * is quantised as in Alg. 2.  The backed-up values are returned in the dense form of Alg. 2's
 * buffer: Bd[m, c] = X[m, c] for the protected channel of each group, +0 elsewhere (Bd is
 * [M, ldb], ldb >= K), and idx[m, g] = j* (may be NULL). */
int ref_quantize_mxfp4_dynamic(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, uint8_t *Xq,
                               uint8_t *Xs, uint16_t *Bd, int64_t ldb, uint8_t *idx) {
    if (M < 0 || K < 0 || K % G || ldx < K || ldb < K) return REF_ERR_ARG;
    if (M == 0 || K == 0) return REF_OK;
    if (!X || !Xq || !Xs || !Bd) return REF_ERR_ARG;
    int64_t Kg = K / G;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        for (int64_t c = 0; c < ldb; ++c) Bd[m * ldb + c] = 0;
        for (int64_t g = 0; g < Kg; ++g) {
            int jstar = 0;
            double best = -1.0;
            for (int j = 0; j < G; ++j) {
                uint16_t h = x[g * G + j];
                if ((h & 0x7F80) == 0x7F80) bad = 1;
                double a = fabs((double)bf16_to_float(h));
                if (a > best) {
                    best = a;
                    jstar = j;
                }
            }
            Bd[m * ldb + g * G + jstar] = x[g * G + jstar];
            if (idx) idx[m * Kg + g] = (uint8_t)jstar;
            double v[G];
            int neg[G];
            double amax = 0.0;
            for (int j = 0; j < G; ++j) {
                uint16_t h = j == jstar ? (uint16_t)0 : x[g * G + j];
                v[j] = (double)bf16_to_float(h);
                neg[j] = (h >> 15) & 1;
                if (fabs(v[j]) > amax) amax = fabs(v[j]);
            }
            int e = mx_shared_exponent(amax);
            Xs[m * Kg + g] = (uint8_t)(e + 127);
            for (int j = 0; j < G; j += 2) {
                int lo = ref_e2m1_encode(ldexp(v[j], -e), neg[j]);
                int hi = ref_e2m1_encode(ldexp(v[j + 1], -e), neg[j + 1]);
                Xq[m * (K / 2) + (g * G + j) / 2] = (uint8_t)(lo | (hi << 4));
            }
        }
    }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}

/* W_L[o, n] = W[n, oidx[o]] for o < K_o, taken from the unquantised weight
 * W[N, K] (bf16 bits, row stride ldw).  W_L is [K_o, N] row-major. */
int ref_gather_wl(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, const int32_t *oidx,
                  int32_t K_o, uint16_t *WL) {
    if (N < 0 || K < 0 || ldw < K || K_o < 0) return REF_ERR_ARG;
    if (K_o == 0 || N == 0) return REF_OK;
    if (!W || !oidx || !WL) return REF_ERR_ARG;
    for (int32_t o = 0; o < K_o; ++o) {
        if (oidx[o] < 0 || oidx[o] >= K) return REF_ERR_TABLE;
        for (int64_t n = 0; n < N; ++n) WL[(int64_t)o * N + n] = W[n * ldw + oidx[o]];
    }
    return REF_OK;
}

/* ---- dual-path GEMM (Eq. dual-path) ------------------------------------ */

/* Y[m, n] = sum_g 2^(Xs[m,g] + Ws[n,g] - 254) * sum_{j<32} e2m1(Xq[m,g,j]) * e2m1(Wq[n,g,j])
 *         + sum_{o<K_o} B[m, o] * W_L[o, n]                       (all in double)
 * Wq[N, K/2], Ws[N, K/32] are the weight quantised along K; W_L is [K_o, N]. */
int ref_dual_gemm(const uint8_t *Xq, const uint8_t *Xs, const uint16_t *B, int64_t ldb,
                  const uint8_t *Wq, const uint8_t *Ws, const uint16_t *WL, int64_t M, int64_t N,
                  int64_t K, int32_t K_o, double *Y, int64_t ldy) {
    if (M < 0 || N < 0 || K < 0 || K % G || K_o < 0 || ldb < K_o || ldy < N) return REF_ERR_ARG;
    if (M == 0 || N == 0) return REF_OK;
    if (!Y || (K && (!Xq || !Xs || !Wq || !Ws)) || (K_o && (!B || !WL))) return REF_ERR_ARG;
    int64_t Kg = K / G;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            /* Path A: low-bit base */
            for (int64_t g = 0; g < Kg; ++g) {
                double s = 0.0;
                for (int j = 0; j < G; ++j) {
                    int64_t k = g * G + j;
                    int qx = (Xq[m * (K / 2) + k / 2] >> (4 * (k & 1))) & 15;
                    int qw = (Wq[n * (K / 2) + k / 2] >> (4 * (k & 1))) & 15;
                    s += ref_e2m1_decode(qx) * ref_e2m1_decode(qw);
                }
                acc += ldexp(s, (int)Xs[m * Kg + g] + (int)Ws[n * Kg + g] - 254);
            }
            /* Path B: high-precision bypass */
            for (int32_t o = 0; o < K_o; ++o)
                acc += (double)bf16_to_float(B[m * ldb + o]) *
                       (double)bf16_to_float(WL[(int64_t)o * N + n]);
            Y[m * ldy + n] = acc;
        }
    }
    return REF_OK;
}

/* E experts; rows [off[e], off[e+1]) of the sorted token list belong to expert
 * e and use its weights.  row_map (may be NULL = identity) names, for each
 * sorted position t, the row of Xq/Xs/B it reads.  Y is indexed by t. */
int ref_grouped_dual_gemm(const uint8_t *Xq, const uint8_t *Xs, const uint16_t *B, int64_t ldb,
                          const int32_t *row_map, const int32_t *off, int32_t E,
                          const uint8_t *Wq, const uint8_t *Ws, const uint16_t *WL, int64_t N,
                          int64_t K, int32_t K_o, double *Y, int64_t ldy) {
    if (E < 0 || !off) return REF_ERR_ARG;
    int64_t Kg = K / G;
    for (int32_t e = 0; e < E; ++e) {
        if (off[e + 1] < off[e]) return REF_ERR_ARG;
        for (int64_t t = off[e]; t < off[e + 1]; ++t) {
            int64_t r = row_map ? row_map[t] : t;
            int rc = ref_dual_gemm(Xq + r * (K / 2), Xs + r * Kg, B ? B + r * ldb : B, ldb,
                                   Wq + (int64_t)e * N * (K / 2), Ws + (int64_t)e * N * Kg,
                                   WL ? WL + (int64_t)e * K_o * N : WL, 1, N, K, K_o,
                                   Y + t * ldy, ldy);
            if (rc) return rc;
        }
    }
    return REF_OK;
}

/* ---- FP8 fallback (Section 3.4) ----------------------------------------- */

/* One row of R[rows, K] (bf16 bits) -> e4m3 codes and one fp32 scale:
 *   amax = max |x|;  rows with amax < 2^-100 (all-zero rows included) use
 *   scale = inv = 1; otherwise scale = amax / 448 and inv = 448 / amax, each
 *   one IEEE single division;  q = e4m3(x * inv), one IEEE single multiply. */
int ref_quantize_fp8_rows(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, uint8_t *X8,
                          float *xs) {
    if (M < 0 || K < 0 || ldx < K) return REF_ERR_ARG;
    if (M == 0) return REF_OK;
    if (!X8 || !xs || (K && !X)) return REF_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            if ((x[k] & 0x7F80) == 0x7F80) bad = 1;
            float a = fabsf(bf16_to_float(x[k]));
            if (a > amax) amax = a;
        }
        volatile float scale = 1.0f, inv = 1.0f;
        if (amax >= 0x1p-100f) {
            scale = amax / 448.0f;
            inv = 448.0f / amax;
        }
        xs[m] = scale;
        for (int64_t k = 0; k < K; ++k) {
            volatile float p = bf16_to_float(x[k]) * inv;
            X8[m * K + k] = (uint8_t)ref_e4m3_encode(p);
        }
    }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}

/* Y[m, n] = xs[m] * ws[n] * sum_k e4m3(X8[m,k]) * e4m3(W8[n,k])   (double) */
int ref_fp8_gemm(const uint8_t *X8, const float *xs, const uint8_t *W8, const float *ws,
                 int64_t M, int64_t N, int64_t K, double *Y, int64_t ldy) {
    if (M < 0 || N < 0 || K < 0 || ldy < N) return REF_ERR_ARG;
    if (M == 0 || N == 0) return REF_OK;
    if (!Y || !xs || !ws || (K && (!X8 || !W8))) return REF_ERR_ARG;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += ref_e4m3_decode(X8[m * K + k]) * ref_e4m3_decode(W8[n * K + k]);
            Y[m * ldy + n] = (double)xs[m] * (double)ws[n] * s;
        }
    }
    return REF_OK;
}

int ref_grouped_fp8_gemm(const uint8_t *X8, const float *xs, const int32_t *off, int32_t E,
                         const uint8_t *W8, const float *ws, int64_t N, int64_t K, double *Y,
                         int64_t ldy) {
    if (E < 0 || !off) return REF_ERR_ARG;
    for (int32_t e = 0; e < E; ++e) {
        if (off[e + 1] < off[e]) return REF_ERR_ARG;
        int64_t t0 = off[e], Me = off[e + 1] - off[e];
        int rc = ref_fp8_gemm(X8 + t0 * K, xs + t0, W8 + (int64_t)e * N * K, ws + (int64_t)e * N,
                              Me, N, K, Y + t0 * ldy, ldy);
        if (rc) return rc;
    }
    return REF_OK;
}

/* ---- MXFP8 form of the fallback (Section 3.4; Section 4.1) --------------- */

/* R[rows, K] (bf16 bits) -> E4M3 codes [rows, K] and E8M0 scales [rows, K/32].
 * Per group of 32: amax = max |x|; shared exponent e = floor(log2 amax) - 8
 * (8 = exponent of the largest E4M3 binade), clamped to [-127, 127];
 * element = e4m3(x / 2^e), nearest even, saturating at +-448.  x / 2^e is
 * exact in double, and ref_e4m3_encode takes a float: the quotient of a bf16
 * by a power of two is a float unless it underflows the float range, where it
 * is below half the smallest E4M3 step anyway and rounds to zero either way. */
int ref_quantize_mxfp8(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, uint8_t *Xq,
                       uint8_t *Xs) {
    if (M < 0 || K < 0 || K % G || ldx < K) return REF_ERR_ARG;
    if (M == 0 || K == 0) return REF_OK;
    if (!X || !Xq || !Xs) return REF_ERR_ARG;
    const int64_t Kg = K / G;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        for (int64_t g = 0; g < Kg; ++g) {
            double amax = 0.0;
            for (int j = 0; j < G; ++j) {
                uint16_t h = x[g * G + j];
                if ((h & 0x7F80) == 0x7F80) bad = 1;
                double a = fabs((double)bf16_to_float(h));
                if (a > amax) amax = a;
            }
            const int e = mx_shared_exponent_for(amax, 8);
            Xs[m * Kg + g] = (uint8_t)(e + 127);
            for (int j = 0; j < G; ++j) {
                double v = ldexp((double)bf16_to_float(x[g * G + j]), -e);
                Xq[m * K + g * G + j] = (uint8_t)ref_e4m3_encode((float)v);
            }
        }
    }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}

/* Y[m, n] = sum_g 2^(Xs[m,g] + Ws[n,g] - 254) * sum_{j<32} e4m3(Xq[m,32g+j]) * e4m3(Wq[n,32g+j])
 * in double. */
int ref_mxfp8_gemm(const uint8_t *Xq, const uint8_t *Xs, const uint8_t *Wq, const uint8_t *Ws,
                   int64_t M, int64_t N, int64_t K, double *Y, int64_t ldy) {
    if (M < 0 || N < 0 || K < 0 || K % G || ldy < N) return REF_ERR_ARG;
    if (M == 0 || N == 0) return REF_OK;
    if (!Y || (K && (!Xq || !Xs || !Wq || !Ws))) return REF_ERR_ARG;
    const int64_t Kg = K / G;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double y = 0.0;
            for (int64_t g = 0; g < Kg; ++g) {
                double s = 0.0;
                for (int j = 0; j < G; ++j)
                    s += ref_e4m3_decode(Xq[m * K + g * G + j]) * ref_e4m3_decode(Wq[n * K + g * G + j]);
                y += ldexp(s, (int)Xs[m * Kg + g] + (int)Ws[n * Kg + g] - 254);
            }
            Y[m * ldy + n] = y;
        }
    }
    return REF_OK;
}

/* ---- 4-bit formats with scale groups of 16 channels --------------------------------------- *
 * Section 3.1 cuts the channels into groups of G in {16, 32, 64} so that they line up
 * with the scale groups of micro-scaling formats; Table 2 has a G = 16 row; the abstract and the conclusion name
 * NVFP4.  The paper gives no arithmetic for either; the readings taken here:
 *   fmt 0 (E8M0 per 16): the MX rule on blocks of 16: shared exponent floor(log2 amax) - 2 as an
 *          E8M0 code, E2M1 elements x / 2^e rounded to nearest even, saturating;
 *   fmt 1 (NVFP4): E2M1 elements, one E4M3 scale per 16 channels, one single-precision scale ts per
 *          tensor (given by the caller: a calibrated constant), every step one IEEE single-precision
 *          operation:  d = 6 * ts;  q = amax / d;  sc = e4m3(q) (nearest even, saturating at 448);
 *          s = value of sc;  den = ts * s;  inv = 1 / den;  element = e2m1(x * inv) (nearest even,
 *          saturating); a block whose scale rounds to zero keeps only the signs of its elements.
 * Everything else is Alg. 2 unchanged: protected channels are copied to B and count as +0 before
 * the scale of their block is computed.  Xs16[M, K/16]: one scale byte per 16 channels, row-major. */
int ref_quantize_fp4_g16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const int32_t *oidx,
                         int32_t K_o, int fmt, float ts, uint8_t *Xq, uint8_t *Xs16, uint16_t *B,
                         int64_t ldb) {
    if (fmt != 0 && fmt != 1) return REF_ERR_ARG;
    if (M < 0 || K < 0 || K % 16 || ldx < K || K_o < 0 || ldb < K_o) return REF_ERR_ARG;
    if (fmt == 1 && !(ts > 0.0f && ts <= FLT_MAX)) return REF_ERR_ARG;
    if (M == 0 || K == 0) return REF_OK;
    if (!X || !Xq || !Xs16 || (K_o && (!oidx || !B))) return REF_ERR_ARG;
    for (int32_t o = 0; o < K_o; ++o)
        if (oidx[o] < 0 || oidx[o] >= K) return REF_ERR_TABLE;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = X + m * ldx;
        uint8_t *removed = (uint8_t *)calloc((size_t)K, 1);
        if (B)
            for (int64_t o = 0; o < ldb; ++o) B[m * ldb + o] = 0;
        for (int32_t o = 0; o < K_o; ++o) {
            B[m * ldb + o] = x[oidx[o]];
            removed[oidx[o]] = 1;
        }
        for (int64_t g = 0; g < K / 16; ++g) {
            float v[16];
            int neg[16];
            float amax = 0.0f;
            for (int j = 0; j < 16; ++j) {
                uint16_t h = removed[g * 16 + j] ? (uint16_t)0 : x[g * 16 + j];
                if ((h & 0x7F80) == 0x7F80) bad = 1;
                v[j] = bf16_to_float(h);
                neg[j] = (h >> 15) & 1;
                if (fabsf(v[j]) > amax) amax = fabsf(v[j]);
            }
            int code[16];
            if (fmt == 0) {
                int e = mx_shared_exponent((double)amax);
                Xs16[m * (K / 16) + g] = (uint8_t)(e + 127);
                for (int j = 0; j < 16; ++j) code[j] = ref_e2m1_encode(ldexp((double)v[j], -e), neg[j]);
            } else {
                volatile float d = 6.0f * ts;
                volatile float q = amax / d;
                int sc = (q <= FLT_MAX) ? ref_e4m3_encode(q) : 0x7E; /* beyond single range: the largest scale */
                sc &= 0x7F;
                Xs16[m * (K / 16) + g] = (uint8_t)sc;
                float sval = (float)ref_e4m3_decode(sc);
                if (sval == 0.0f) {
                    for (int j = 0; j < 16; ++j) code[j] = neg[j] ? 8 : 0;
                } else {
                    volatile float den = ts * sval;
                    volatile float inv = 1.0f / den;
                    for (int j = 0; j < 16; ++j) {
                        volatile float w = v[j] * inv;
                        code[j] = (fabsf(w) <= FLT_MAX) ? ref_e2m1_encode((double)w, neg[j]) : (neg[j] ? 15 : 7);
                    }
                }
            }
            for (int j = 0; j < 16; j += 2)
                Xq[m * (K / 2) + (g * 16 + j) / 2] = (uint8_t)(code[j] | (code[j + 1] << 4));
        }
        free(removed);
    }
    return bad ? REF_ERR_NONFINITE : REF_OK;
}

static double scale16_value(int fmt, int code) {
    return fmt == 0 ? ldexp(1.0, code - 127) : ref_e4m3_decode(code & 0x7F);
}

/* The dual-path layer on those operands (Eq. dual-path with the scale of a block of 16):
 *   Y[m,n] = xts * wts * sum_b s(Xs16[m,b]) * s(Ws16[n,b]) * sum_{j<16} e2m1(Xq[m,16b+j]) * e2m1(Wq[n,16b+j])
 *          + sum_{o<K_o} B[m,o] * W_L[o,n]            (xts = wts = 1 for fmt 0), all in double. */
int ref_dual_gemm_g16(const uint8_t *Xq, const uint8_t *Xs16, float xts, const uint16_t *B, int64_t ldb,
                      const uint8_t *Wq, const uint8_t *Ws16, float wts, const uint16_t *WL, int64_t M,
                      int64_t N, int64_t K, int32_t K_o, int fmt, double *Y, int64_t ldy) {
    if ((fmt != 0 && fmt != 1) || M < 0 || N < 0 || K < 0 || K % 16 || K_o < 0 || ldy < N) return REF_ERR_ARG;
    if (M == 0 || N == 0) return REF_OK;
    if (!Y || (K && (!Xq || !Xs16 || !Wq || !Ws16)) || (K_o && (!B || !WL || ldb < K_o))) return REF_ERR_ARG;
    const double ts = fmt == 1 ? (double)xts * (double)wts : 1.0;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t b = 0; b < K / 16; ++b) {
                double part = 0.0;
                for (int j = 0; j < 16; ++j) {
                    int64_t k = b * 16 + j;
                    int cx = (Xq[m * (K / 2) + k / 2] >> (4 * (k & 1))) & 15;
                    int cw = (Wq[n * (K / 2) + k / 2] >> (4 * (k & 1))) & 15;
                    part += ref_e2m1_decode(cx) * ref_e2m1_decode(cw);
                }
                acc += part * scale16_value(fmt, Xs16[m * (K / 16) + b]) * scale16_value(fmt, Ws16[n * (K / 16) + b]);
            }
            acc *= ts;
            for (int32_t o = 0; o < K_o; ++o)
                acc += (double)bf16_to_float(B[m * ldb + o]) * (double)bf16_to_float(WL[(int64_t)o * N + n]);
            Y[m * ldy + n] = acc;
        }
    return REF_OK;
}

/* ---- offline profiling (Section 2, Alg. 1) ------------------------------- */

/* Eq. 1: T = alpha / (S*H) * sum |x|, accumulated in double in row-major order. */
int ref_profile_threshold(const uint16_t *X, int64_t S, int64_t H, int64_t ldx, double alpha,
                          double *T) {
    if (!X || !T || S <= 0 || H <= 0 || ldx < H) return REF_ERR_ARG;
    double sum = 0.0;
    for (int64_t s = 0; s < S; ++s)
        for (int64_t j = 0; j < H; ++j) {
            const uint16_t h = X[s * ldx + j];
            if ((h & 0x7F80u) == 0x7F80u) return REF_ERR_NONFINITE;
            sum += fabs((double)bf16_to_float(h));
        }
    *T = alpha * (sum / ((double)S * (double)H));
    return REF_OK;
}

/* Eq. 2 and Eq. 3 for every token s and group k of Gp channels: j* = argmax_j |x[s, k*Gp + j]|
 * (the lowest j among equal magnitudes); when |x[s, k*Gp + j*]| > T the token belongs to S_k and
 * hist[k][j*] grows by one.  Counts are added to what hist already holds, so a calibration set
 * can be fed in pieces. */
int ref_profile_hist(const uint16_t *X, int64_t S, int64_t H, int64_t ldx, int32_t Gp, double T,
                     uint32_t *hist) {
    if (!X || !hist || S < 0 || H < 0 || Gp <= 0 || H % Gp || ldx < H) return REF_ERR_ARG;
    for (int64_t s = 0; s < S; ++s)
        for (int64_t k = 0; k < H / Gp; ++k) {
            int jstar = 0;
            double best = -1.0;
            for (int j = 0; j < Gp; ++j) {
                const uint16_t h = X[s * ldx + k * Gp + j];
                if ((h & 0x7F80u) == 0x7F80u) return REF_ERR_NONFINITE;
                const double a = fabs((double)bf16_to_float(h));
                if (a > best) {
                    best = a;
                    jstar = j;
                }
            }
            if (best > T) hist[k * Gp + jstar] += 1;
        }
    return REF_OK;
}

/* Alg. 1's table entry and Eq. 4 from the counts of one layer and position.
 *   table[k][0..R-1]  the R local indices with the largest counts, most frequent first (equal
 *                     counts: lower index first); only indices with a count above zero; the
 *                     rest -1.  R = 1 is the table of Alg. 1: the mode, or -1 for an empty set.
 *   n_total[k] = |S_k|, n_hit[k] = the largest count, density[k] = n_hit / n_total (0 when the
 *   set is empty); *cbar = mean of density over the groups whose set is not empty (0 when all
 *   are empty). */
int ref_profile_table(const uint32_t *hist, int32_t Kg, int32_t Gp, int32_t R, int16_t *table,
                      uint32_t *n_total, uint32_t *n_hit, double *density, double *cbar) {
    if (!hist || Kg < 0 || Gp <= 0 || R < 0 || (R && !table)) return REF_ERR_ARG;
    double dsum = 0.0;
    int64_t nonempty = 0;
    for (int32_t k = 0; k < Kg; ++k) {
        const uint32_t *h = hist + (int64_t)k * Gp;
        uint64_t total = 0;
        uint32_t top = 0;
        for (int j = 0; j < Gp; ++j) {
            total += h[j];
            if (h[j] > top) top = h[j];
        }
        if (n_total) n_total[k] = (uint32_t)total;
        if (n_hit) n_hit[k] = top;
        const double c = total ? (double)top / (double)total : 0.0;
        if (density) density[k] = c;
        if (total) {
            dsum += c;
            ++nonempty;
        }
        /* selection of the R most frequent indices, one at a time */
        for (int32_t r = 0; r < R; ++r) {
            int pick = -1;
            for (int j = 0; j < Gp; ++j) {
                if (h[j] == 0) continue;
                int taken = 0;
                for (int32_t q = 0; q < r; ++q)
                    if (table[(int64_t)k * R + q] == j) taken = 1;
                if (taken) continue;
                if (pick < 0 || h[j] > h[pick]) pick = j;
            }
            table[(int64_t)k * R + r] = (int16_t)pick;
        }
    }
    if (cbar) *cbar = nonempty ? dsum / (double)nonempty : 0.0;
    return REF_OK;
}

/* threads the parallel loops above actually use */
int ref_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
