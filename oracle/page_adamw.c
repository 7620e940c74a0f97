/*
 * ORACLE — TEST INFRASTRUCTURE ONLY.  Never linked, imported or called by the product path.
 *
 * Plain scalar double-precision definition of the page-granular mixed-precision AdamW update of
 * Angel-PTM's optimizer step: FP32 master parameter / momentum / variance updated element-wise
 * from 16-bit gradients and cast back to 16-bit parameters (Sec. 2 "Mixed Precision Training";
 * Sec. 2.2 "master parameter, momentum, variance"; Alg. 2 "Update p32, m32, v32 via g'16" and
 * "p'16 <- cast(p32)"; Sec. 4.3 last paragraph: the update is element-wise, hence page-level).
 * The paper names the optimizer (Adam, Kingma & Ba) without printing its equations; the reading
 * used here (decoupled weight decay, bias correction, eps added outside the root, per-page L2
 * clipping, skip of gradient-free pages, 16-bit format = bf16 as in Sec. 6.1) is this build's and
 * is pinned by tests against closed forms and against torch.optim.AdamW in float64.
 *
 * No blocking, no vectorisation, no reordering: one loop per step of the definition.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

typedef struct {
    double lr, beta1, beta2, eps, weight_decay;
    double max_grad_norm; /* <= 0: clipping off */
    int32_t skip_mode;    /* 0: every page is updated; 1: pages whose gradient is all zero are untouched */
    int32_t round_state_f32; /* diagnostic: round p, m, v to fp32 after every step */
} oracle_hyper;

static double bf16_to_double(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f; /* exact */
}

/* Round-to-nearest-even of an fp32 bit pattern to bf16, written on the integer representation.
 * Pinned on every fp32 pattern against a library cast; for NaN inputs the pins fix that the result
 * is a NaN of the same sign -- which payload bits it carries is parity unpinned. */
uint16_t oracle_bf16_rne(uint32_t u) {
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) /* NaN: keep sign/payload top bits, force quiet bit */
        return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

/* Step 1 and 3 of the page definition: any-nonzero test on magnitude bits, sum of squares. */
void oracle_page_reduce(const uint16_t* g16, int64_t n, int32_t* nz, double* sumsq) {
    int32_t any = 0;
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if ((g16[i] & 0x7FFFu) != 0) any = 1;
        double g = bf16_to_double(g16[i]);
        s += g * g;
    }
    *nz = any;
    *sumsq = s;
}

/*
 * One AdamW step on the n used elements of one page, global step t >= 1.
 * p, m, v: double state (in/out).  p16: bf16 bits (out, untouched if the page is skipped).
 * norm_out: fp32(sqrt(sum g^2)) (0 for a skipped page).  skip_out: 1 if skipped.
 * Returns 0, or -1 on t < 1.
 */
int oracle_page_adamw(double* p, double* m, double* v, uint16_t* p16, const uint16_t* g16,
                      int64_t n, int64_t t, const oracle_hyper* h, float* norm_out,
                      uint8_t* skip_out) {
    if (t < 1) return -1;
    int32_t nz;
    double sumsq;
    oracle_page_reduce(g16, n, &nz, &sumsq);
    if (h->skip_mode == 1 && !nz) {
        *skip_out = 1;
        *norm_out = 0.0f;
        return 0;
    }
    *skip_out = 0;
    double norm = sqrt(sumsq);
    *norm_out = (float)norm;
    double s = 1.0;
    if (h->max_grad_norm > 0.0) {
        s = h->max_grad_norm / (norm + 1e-6);
        if (s > 1.0) s = 1.0;
    }
    const double bc1 = 1.0 - pow(h->beta1, (double)t);
    const double bc2 = 1.0 - pow(h->beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double g = s * bf16_to_double(g16[i]);
        double mi = h->beta1 * m[i] + (1.0 - h->beta1) * g;
        double vi = h->beta2 * v[i] + (1.0 - h->beta2) * g * g;
        double mhat = mi / bc1;
        double vhat = vi / bc2;
        double pi = p[i] * (1.0 - h->lr * h->weight_decay) - h->lr * mhat / (sqrt(vhat) + h->eps);
        if (h->round_state_f32) {
            mi = (double)(float)mi;
            vi = (double)(float)vi;
            pi = (double)(float)pi;
        }
        m[i] = mi;
        v[i] = vi;
        p[i] = pi;
        float pf = (float)pi; /* round to nearest even, then a second rounding to bf16 */
        uint32_t u;
        memcpy(&u, &pf, 4);
        p16[i] = oracle_bf16_rne(u);
    }
    return 0;
}

/* Vector form of the cast, for tests: fp32 bit patterns in, bf16 bit patterns out. */
void oracle_bf16_rne_array(const uint32_t* in, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_bf16_rne(in[i]);
}
