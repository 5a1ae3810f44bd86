/*
 * CPU oracle for the RT-Lynx hot path (test infrastructure, NOT a product path).
 *
 * Plain scalar C, one obvious loop nest per step, written from the paper's method section:
 *   Alg. 1 step "X~ <- TopK(X)"           -> orc_topk24      (2:4 magnitude Top-K along D_in)
 *   Alg. 1 step "s <- sqrt(|X|^2/(|X~|^2+eps)), S(X) <- s*X~"
 *     and the unnumbered equation of "Norm-Compensated Sparsification"
 *                                          -> orc_scales, orc_apply
 *   App. A (A_nnz + 2-bit index per kept element)
 *                                          -> orc_pack, orc_unpack
 *   Alg. 1 step "Y_s <- S(X) W^T", Eq. (sparse_activation); optional "+ b" of Alg. 2
 *                                          -> orc_linear   (fp32 triple loop on the masked input)
 *   Eq. (linear_layer) Y = X W^T           -> orc_linear on the un-masked input
 *   App. RFE metric                        -> orc_rfe
 *   Eq. (sparse+lora), Alg. 1 "Y_r <- X (L_A L_B)^T", "Y <- Y_s + Y_r"
 *                                          -> orc_lora_delta, orc_linear_f32w, orc_add
 *   Implementation details, "orthogonal validation with FP8 quantization" (symmetric FP8
 *     quantisation of the activations, weights cast directly to FP8) on the 2:4 FP8 format of
 *     the App. A table of sparse-tensor-core formats
 *                                          -> orc_e4m3_encode / _decode, orc_apply_fp8, orc_pack8
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares no code, tables or constants with the HIP library.
 *
 * Readings of points the paper leaves open (each also listed in the design notes):
 *  - "largest" means largest magnitude (Alg. 2 wording); ties keep the lower index.
 *  - magnitude is compared on the bf16 bit pattern with the sign bit cleared, so -0 == +0,
 *    inf > finite, and NaN patterns rank above inf (NaNs are kept and propagate).
 *  - scope of the norms in s: GROUP (the 1x4 group of the method section, default),
 *    ROW (one token), TENSOR (Alg. 1 read literally), NONE.
 *  - GROUP arithmetic is fp32 in a fixed order (the order is part of the definition because
 *    the result is re-rounded to bf16 for the matrix unit); ROW/TENSOR norms are summed in fp64.
 *  - eps = 1e-8 sits inside the square root, added to the kept norm.
 *  - FP8 is the 8-bit E4M3 format without infinities (bias 7, largest finite 448, S.1111.111 =
 *    NaN); conversion is round-to-nearest-even and saturating: |v| >= 448 and +-inf give +-448,
 *    NaN gives 0x7F. Weights are cast as they are; activations are divided by one caller-supplied
 *    positive scale ("symmetric": no zero point) after selection and compensation, so every
 *    kept value is rounded once: q = e4m3((s * x) * (1 / x_scale)), both products in fp32.
 */
#include <stdint.h>
#include <string.h>
#include <math.h>
#include <stddef.h>

enum { ORC_NONE = 0, ORC_GROUP = 1, ORC_ROW = 2, ORC_TENSOR = 3 };

static float bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even fp32 -> bf16; NaN stays NaN (quiet bit forced). */
static uint16_t f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

float    orc_bf16_to_f32(uint16_t h) { return bf16_to_f32(h); }
uint16_t orc_f32_to_bf16(float f)    { return f32_to_bf16(f); }

/* TopK(.) of Alg. 1: for every row and every aligned group of 4 along D_in, keep[m,k]=1 for the
 * two entries of largest magnitude, else 0. Element i is kept iff fewer than two elements of its
 * group beat it, where j beats i when |x_j| > |x_i|, or |x_j| == |x_i| and j < i. */
int orc_topk24(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* keep) {
    if (K % 4 != 0) return 1;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < K / 4; ++g) {
            const uint16_t* x = X + m * ldx + 4 * g;
            for (int i = 0; i < 4; ++i) {
                unsigned ai = x[i] & 0x7FFFu;
                int beaten = 0;
                for (int j = 0; j < 4; ++j) {
                    unsigned aj = x[j] & 0x7FFFu;
                    if (aj > ai || (aj == ai && j < i)) ++beaten;
                }
                keep[m * K + 4 * g + i] = (uint8_t)(beaten < 2);
            }
        }
    }
    return 0;
}

/* s of Alg. 1 / the norm-compensation equation, one value per scope:
 *   GROUP -> s[M*K/4], ROW -> s[M], TENSOR -> s[1], NONE -> nothing written.
 * GROUP: fp32, num = ((x0^2+x1^2)+x2^2)+x3^2, den = (ka^2+kb^2)+eps with ka the lower-index kept
 * value, s = sqrtf(num/den). ROW/TENSOR: the same quotient with fp64 sums in index order. */
int orc_scales(const uint16_t* X, const uint8_t* keep, int64_t M, int64_t K, int64_t ldx,
               int scope, float eps, float* s) {
    if (K % 4 != 0) return 1;
    if (scope == ORC_NONE) return 0;
    if (scope == ORC_GROUP) {
        for (int64_t m = 0; m < M; ++m)
            for (int64_t g = 0; g < K / 4; ++g) {
                const uint16_t* x = X + m * ldx + 4 * g;
                const uint8_t* kp = keep + m * K + 4 * g;
                float num = 0.0f, den = 0.0f;
                for (int i = 0; i < 4; ++i) {
                    float v = bf16_to_f32(x[i]);
                    float sq = v * v;
                    num = num + sq;
                    if (kp[i]) den = den + sq;
                }
                den = den + eps;
                s[m * (K / 4) + g] = sqrtf(num / den);
            }
        return 0;
    }
    double tnum = 0.0, tden = 0.0;
    for (int64_t m = 0; m < M; ++m) {
        double num = 0.0, den = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = (double)bf16_to_f32(X[m * ldx + k]);
            num += v * v;
            if (keep[m * K + k]) den += v * v;
        }
        if (scope == ORC_ROW) s[m] = (float)sqrt(num / (den + (double)eps));
        tnum += num;
        tden += den;
    }
    if (scope == ORC_TENSOR) s[0] = (float)sqrt(tnum / (tden + (double)eps));
    return 0;
}

/* S(X) = s * X~ as a dense masked fp32 matrix S[M,K] (zeros where dropped).
 * operand_round != 0 re-rounds every product to bf16 (RNE), which is what a bf16 matrix unit
 * is fed; Sb (nullable) receives those bf16 bit patterns (only meaningful with operand_round). */
int orc_apply(const uint16_t* X, const uint8_t* keep, const float* s, int64_t M, int64_t K,
              int64_t ldx, int scope, int operand_round, float* S, uint16_t* Sb) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            float out = 0.0f;
            uint16_t outb = 0;
            if (keep[m * K + k]) {
                float v = bf16_to_f32(X[m * ldx + k]);
                float sc = 1.0f;
                if (scope == ORC_GROUP) sc = s[m * (K / 4) + k / 4];
                else if (scope == ORC_ROW) sc = s[m];
                else if (scope == ORC_TENSOR) sc = s[0];
                out = (scope == ORC_NONE) ? v : sc * v;
                outb = f32_to_bf16(out);
                if (operand_round) out = bf16_to_f32(outb);
            }
            S[m * K + k] = out;
            if (Sb) Sb[m * K + k] = outb;
        }
    return 0;
}

/* Compressed operand of App. A: per group the two kept values in ascending position order plus
 * their 2-bit positions. vals[M,K/2] bf16 bits; meta[M,K/8] bytes, group g of a row in nibble
 * (g & 1) of byte g/2, nibble = pos0 | pos1 << 2. D is the dense bf16 matrix whose kept entries
 * are stored (X itself, or the rounded S(X)). */
int orc_pack(const uint16_t* D, int64_t ldd, const uint8_t* keep, int64_t M, int64_t K,
             uint16_t* vals, uint8_t* meta) {
    if (K % 8 != 0) return 1;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t b = 0; b < K / 8; ++b) meta[m * (K / 8) + b] = 0;
        for (int64_t g = 0; g < K / 4; ++g) {
            int pos[2], n = 0;
            for (int i = 0; i < 4; ++i)
                if (keep[m * K + 4 * g + i]) { if (n < 2) pos[n] = i; ++n; }
            if (n != 2) return 2;
            vals[m * (K / 2) + 2 * g + 0] = D[m * ldd + 4 * g + pos[0]];
            vals[m * (K / 2) + 2 * g + 1] = D[m * ldd + 4 * g + pos[1]];
            unsigned nib = (unsigned)pos[0] | ((unsigned)pos[1] << 2);
            meta[m * (K / 8) + g / 2] |= (uint8_t)(nib << (4 * (g & 1)));
        }
    }
    return 0;
}

/* Inverse of orc_pack: dense bf16 [M,K] with zeros at the dropped positions. */
int orc_unpack(const uint16_t* vals, const uint8_t* meta, int64_t M, int64_t K, uint16_t* D) {
    if (K % 8 != 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t g = 0; g < K / 4; ++g) {
            unsigned nib = (meta[m * (K / 8) + g / 2] >> (4 * (g & 1))) & 0xFu;
            for (int i = 0; i < 4; ++i) D[m * K + 4 * g + i] = 0;
            D[m * K + 4 * g + (nib & 3u)] = vals[m * (K / 2) + 2 * g + 0];
            D[m * K + 4 * g + (nib >> 2)] = vals[m * (K / 2) + 2 * g + 1];
        }
    return 0;
}

/* Y[m,n] = sum_k S[m,k] * W[n,k] (+ bias[n]); fp32 products and fp32 accumulation with k
 * ascending, zeros of S included. W and bias are bf16 bit patterns. Rows m in [m0, m1). */
int orc_linear(const float* S, const uint16_t* W, const uint16_t* bias, int64_t M, int64_t N,
               int64_t K, int64_t ldw, int64_t m0, int64_t m1, float* Y) {
    if (m0 < 0 || m1 > M || m0 > m1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = m0; m < m1; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float acc = 0.0f;
            for (int64_t k = 0; k < K; ++k) acc = acc + S[m * K + k] * bf16_to_f32(W[n * ldw + k]);
            if (bias) acc = acc + bf16_to_f32(bias[n]);
            Y[m * N + n] = acc;
        }
    return 0;
}

/* LoRA product of Eq. (sparse+lora): D[n,k] = sum_r L_A[n,r] * L_B[r,k], fp32, r ascending.
 * L_A [N,R] and L_B [R,K] are bf16 bit patterns, row-major. */
int orc_lora_delta(const uint16_t* LA, const uint16_t* LB, int64_t N, int64_t K, int64_t R, float* D) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            float acc = 0.0f;
            for (int64_t r = 0; r < R; ++r)
                acc = acc + bf16_to_f32(LA[n * R + r]) * bf16_to_f32(LB[r * K + k]);
            D[n * K + k] = acc;
        }
    return 0;
}

/* Y[m,n] = sum_k A[m,k] * Wf[n,k] with an fp32 weight matrix (the LoRA product above), fp32,
 * k ascending. Rows m in [m0, m1). */
int orc_linear_f32w(const float* A, const float* Wf, int64_t M, int64_t N, int64_t K,
                    int64_t m0, int64_t m1, float* Y) {
    if (m0 < 0 || m1 > M || m0 > m1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = m0; m < m1; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float acc = 0.0f;
            for (int64_t k = 0; k < K; ++k) acc = acc + A[m * K + k] * Wf[n * K + k];
            Y[m * N + n] = acc;
        }
    return 0;
}

/* out = a + b elementwise in fp32 (Alg. 1 "Y <- Y_s + Y_r"). */
int orc_add(const float* a, const float* b, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = a[i] + b[i];
    return 0;
}

/* ---- FP8 (E4M3, finite-only variant) ------------------------------------------------------ */

/* Value of an E4M3 code: S.EEEE.MMM, bias 7; E = 0 is subnormal (M * 2^-9); 0x7F / 0xFF are NaN. */
static float e4m3_to_f32(uint8_t c) {
    int e = (c >> 3) & 0xF, m = c & 7;
    float v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexpf((float)m, -9);
    else v = ldexpf((float)(8 + m), e - 7 - 3);
    return (c & 0x80) ? -v : v;
}

/* fp32 -> E4M3, round-to-nearest-even, saturating. */
static uint8_t f32_to_e4m3(float f) {
    uint8_t sign = signbit(f) ? 0x80 : 0x00;
    float a = fabsf(f);
    int e;
    float q, lo, frac;
    int r;
    if (isnan(f)) return 0x7F;
    if (a >= 448.0f) return (uint8_t)(sign | 0x7E);
    if (a == 0.0f) return sign;
    (void)frexpf(a, &e);          /* a = m * 2^e, m in [0.5, 1)  ->  a in [2^(e-1), 2^e) */
    e -= 1;
    if (e < -6) e = -6;           /* below the smallest normal the quantum stays 2^-9 */
    q = ldexpf(a, 3 - e);         /* exact: in units of the quantum; [8,16) normal, [0,8) subnormal */
    lo = floorf(q);
    frac = q - lo;                /* exact */
    r = (int)lo;
    if (frac > 0.5f || (frac == 0.5f && (r & 1))) r += 1;
    if (r == 16) { r = 8; e += 1; }
    if (r < 8) return (uint8_t)(sign | r);                       /* subnormal (e == -6) or zero */
    return (uint8_t)(sign | ((e + 7) << 3) | (r - 8));
}

int orc_e4m3_encode(const float* in, int64_t n, uint8_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = f32_to_e4m3(in[i]);
    return 0;
}
int orc_e4m3_decode(const uint8_t* in, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = e4m3_to_f32(in[i]);
    return 0;
}

/* FP8 form of S(X): Q[M,K] holds the E4M3 code of (s * x) * (1 / x_scale) at kept positions and
 * 0 elsewhere; s is the GROUP factor (scope GROUP) or 1 (ROW / TENSOR factors are constant along
 * the contraction and multiply Y instead, NONE has none). */
int orc_apply_fp8(const uint16_t* X, const uint8_t* keep, const float* s, int64_t M, int64_t K,
                  int64_t ldx, int scope, float x_scale, uint8_t* Q) {
    const float inv = 1.0f / x_scale;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t q = 0;
            if (keep[m * K + k]) {
                float v = bf16_to_f32(X[m * ldx + k]);
                if (scope == ORC_GROUP) v = s[m * (K / 4) + k / 4] * v;
                v = v * inv;
                q = f32_to_e4m3(v);
            }
            Q[m * K + k] = q;
        }
    return 0;
}

/* orc_pack for one-byte elements: vals8[M,K/2], meta as in orc_pack. */
int orc_pack8(const uint8_t* D, const uint8_t* keep, int64_t M, int64_t K, uint8_t* vals, uint8_t* meta) {
    if (K % 8 != 0) return 1;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t b = 0; b < K / 8; ++b) meta[m * (K / 8) + b] = 0;
        for (int64_t g = 0; g < K / 4; ++g) {
            int pos[2], n = 0;
            for (int i = 0; i < 4; ++i)
                if (keep[m * K + 4 * g + i]) { if (n < 2) pos[n] = i; ++n; }
            if (n != 2) return 2;
            vals[m * (K / 2) + 2 * g + 0] = D[m * K + 4 * g + pos[0]];
            vals[m * (K / 2) + 2 * g + 1] = D[m * K + 4 * g + pos[1]];
            unsigned nib = (unsigned)pos[0] | ((unsigned)pos[1] << 2);
            meta[m * (K / 8) + g / 2] |= (uint8_t)(nib << (4 * (g & 1)));
        }
    }
    return 0;
}

/* bf16 bits -> fp32 matrix (used to feed orc_linear with the un-sparsified X: Eq. linear_layer). */
int orc_widen(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, float* out) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) out[m * K + k] = bf16_to_f32(X[m * ldx + k]);
    return 0;
}

/* fp32 -> bf16 RNE over an array (the store path of the epilogue). */
int orc_round_bf16(const float* in, int64_t n, uint16_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = f32_to_bf16(in[i]);
    return 0;
}

/* Relative Frobenius error ||A - B||_F / ||A||_F (appendix RFE metric), fp64 sums. */
double orc_rfe(const float* A, const float* B, int64_t n) {
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double d = (double)A[i] - (double)B[i];
        num += d * d;
        den += (double)A[i] * (double)A[i];
    }
    return den > 0.0 ? sqrt(num / den) : 0.0;
}

int orc_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = __builtin_omp_get_num_threads();
    }
#endif
    return n;
}
