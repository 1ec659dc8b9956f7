/*
 * ffsnap_oracle.c -- plain, slow, single-threaded CPU reference for the snapshot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product library links, loads or calls this file;
 * it shares no code, table or constant with the GPU library.  It exists so that the GPU path
 * can be compared with something a reader can check by eye.
 *
 * What it computes (FFTrainer, section 4.2 "Checkpoint razor and fast snapshot": every
 * iteration the unique training state of one worker -- a list of tensors -- is copied, without
 * any serialisation, into one pre-allocated contiguous buffer; section 3.1 steps 5-6 and
 * section 3.3: on failover a newcomer receives that buffer and loads its tensors from it;
 * section 6.2: the optimizer state is snapshotted immediately after each update):
 *
 *   stream   T = b_0 || b_1 || ... || b_{n-1}      raw little-endian bytes of the segments,
 *                                                  caller's order, no padding between them
 *   buffer     = T || 0x00^(n_chunks*C - |T|)      n_chunks = ceil(|T| / C)
 *   crc[j]     = CRC32C(buffer[jC : (j+1)C])       over all C bytes, zero tail included
 *   restore    : crc'[j] recomputed; bad[j] = crc'[j] != crc[j]; n_bad = sum(bad);
 *                every segment i gets buffer[off_i : off_i + L_i], good chunk or bad
 *   adam       : one AdamW step in fp32 with a fixed operation order (below), in place,
 *                NaN results stored in one canonical form, followed by pack of the updated state
 *
 * The paper fixes none of chunking, checksum or optimizer arithmetic; the definitions above
 * are the readings taken.  CRC32C is the Castagnoli CRC of iSCSI (RFC 3720 section 12.1):
 * polynomial 0x1EDC6F41, reflected in and out, initial value and final XOR 0xFFFFFFFF.
 *
 * Parity pins (tests/test_oracle_*.py): RFC 3720 B.4 vectors and the "123456789" check value;
 * polynomial long division over GF(2) with Python integers; combine identity by brute force;
 * numpy.concatenate for pack; round trip for restore; torch.optim.AdamW in float64 and closed
 * -form special cases for Adam; torch's bf16 cast for the rounding; numpy's IEEE conversions
 * for the fp16 variant, and bit equality with the bf16 step on shared values.  Nothing here is
 * unpinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define POLY_REFLECTED 0x82F63B78u /* 0x1EDC6F41 bit-reversed */

/* ---- CRC32C ---------------------------------------------------------------------------- */

/* One byte through the reflected shift register: the definition, bit by bit. */
static uint32_t reg_step_byte(uint32_t c, uint8_t b)
{
    c ^= b;
    for (int k = 0; k < 8; k++)
        c = (c >> 1) ^ ((c & 1u) ? POLY_REFLECTED : 0u);
    return c;
}

/* Register update over n bytes with neither initial value nor final XOR applied. */
uint32_t orc_crc_reg(uint32_t c, const uint8_t *p, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++)
        c = reg_step_byte(c, p[i]);
    return c;
}

/* CRC32C straight from the definition. */
uint32_t orc_crc32c_bitwise(const uint8_t *p, uint64_t n)
{
    return orc_crc_reg(0xFFFFFFFFu, p, n) ^ 0xFFFFFFFFu;
}

/* The same function with the inner 8 steps tabulated per byte value (table built from the
 * bitwise step on first use).  Used for the large buffers; checked against the bitwise form. */
static uint32_t byte_table[256];
static int byte_table_ready = 0;

static void build_byte_table(void)
{
    for (uint32_t b = 0; b < 256; b++)
        byte_table[b] = reg_step_byte(0u, (uint8_t)b);
    byte_table_ready = 1;
}

void orc_init(void)
{
    if (!byte_table_ready)
        build_byte_table();
}

uint32_t orc_crc32c(const uint8_t *p, uint64_t n)
{
    orc_init();
    uint32_t c = 0xFFFFFFFFu;
    for (uint64_t i = 0; i < n; i++)
        c = (c >> 8) ^ byte_table[(c ^ p[i]) & 0xFFu];
    return c ^ 0xFFFFFFFFu;
}

/* shift(c, n): run the register from c over n zero bytes (no init, no final XOR).  In
 * polynomial terms: multiply by x^(8n) modulo the generator. */
uint32_t orc_crc_shift(uint32_t c, uint64_t nbytes)
{
    for (uint64_t i = 0; i < nbytes; i++)
        c = reg_step_byte(c, 0);
    return c;
}

/* crc(A || B) from crc(A), crc(B) and |B| for the standard CRC (init and final XOR applied). */
uint32_t orc_crc32c_combine(uint32_t crc_a, uint32_t crc_b, uint64_t len_b)
{
    return orc_crc_shift(crc_a, len_b) ^ crc_b;
}

/* ---- pack / restore -------------------------------------------------------------------- */

static uint64_t total_bytes(const uint64_t *nbytes, uint64_t n_segs)
{
    uint64_t t = 0;
    for (uint64_t i = 0; i < n_segs; i++)
        t += nbytes[i];
    return t;
}

uint64_t orc_num_chunks(const uint64_t *nbytes, uint64_t n_segs, uint64_t chunk_bytes)
{
    uint64_t t = total_bytes(nbytes, n_segs);
    return (t + chunk_bytes - 1) / chunk_bytes;
}

/* Fill buffer[lo:hi) (stream coordinates) from the segments; zero beyond the payload. */
static void gather_range(const uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
                         uint8_t *buffer, uint64_t lo, uint64_t hi)
{
    uint64_t off = 0; /* stream offset of segment i */
    memset(buffer + lo, 0, hi - lo);
    for (uint64_t i = 0; i < n_segs; i++) {
        uint64_t a = off, b = off + nbytes[i]; /* segment i occupies [a, b) */
        uint64_t s = a > lo ? a : lo, e = b < hi ? b : hi;
        if (s < e)
            memcpy(buffer + s, ptrs[i] + (s - a), e - s);
        off = b;
    }
}

/* Pack chunks [j0, j1): buffer bytes and crcs[j].  `buffer` and `crcs` address the WHOLE
 * snapshot (chunk j lives at buffer + j*C), so disjoint ranges can be packed independently. */
void orc_pack_chunks(const uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
                     uint64_t chunk_bytes, uint8_t *buffer, uint32_t *crcs,
                     uint64_t j0, uint64_t j1)
{
    for (uint64_t j = j0; j < j1; j++) {
        gather_range(ptrs, nbytes, n_segs, buffer, j * chunk_bytes, (j + 1) * chunk_bytes);
        crcs[j] = orc_crc32c(buffer + j * chunk_bytes, chunk_bytes);
    }
}

void orc_pack(const uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
              uint64_t chunk_bytes, uint8_t *buffer, uint32_t *crcs)
{
    orc_pack_chunks(ptrs, nbytes, n_segs, chunk_bytes, buffer, crcs, 0,
                    orc_num_chunks(nbytes, n_segs, chunk_bytes));
}

/* Verify chunks [j0, j1): bad[j] in {0,1}; returns how many of them are bad. */
uint64_t orc_verify_chunks(const uint8_t *buffer, const uint32_t *crcs, uint64_t chunk_bytes,
                           uint32_t *bad, uint64_t j0, uint64_t j1)
{
    uint64_t n_bad = 0;
    for (uint64_t j = j0; j < j1; j++) {
        bad[j] = (orc_crc32c(buffer + j * chunk_bytes, chunk_bytes) != crcs[j]) ? 1u : 0u;
        n_bad += bad[j];
    }
    return n_bad;
}

/* Scatter segments [i0, i1) out of the buffer. */
void orc_scatter_segments(uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
                          const uint8_t *buffer, uint64_t i0, uint64_t i1)
{
    uint64_t off = 0;
    for (uint64_t i = 0; i < n_segs; i++) {
        if (i >= i0 && i < i1 && nbytes[i])
            memcpy(ptrs[i], buffer + off, nbytes[i]);
        off += nbytes[i];
    }
}

/* Restore: verify every chunk, then scatter every segment (from good and bad chunks alike). */
uint64_t orc_restore(uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
                     uint64_t chunk_bytes, const uint8_t *buffer, const uint32_t *crcs,
                     uint32_t *bad)
{
    uint64_t n_chunks = orc_num_chunks(nbytes, n_segs, chunk_bytes);
    uint64_t n_bad = orc_verify_chunks(buffer, crcs, chunk_bytes, bad, 0, n_chunks);
    orc_scatter_segments(ptrs, nbytes, n_segs, buffer, 0, n_segs);
    return n_bad;
}

/* Copy buffer[lo:hi) (stream coordinates, hi <= payload) out to the segments it covers. */
static void scatter_range(uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
                          const uint8_t *buffer, uint64_t lo, uint64_t hi)
{
    uint64_t off = 0;
    for (uint64_t i = 0; i < n_segs; i++) {
        uint64_t a = off, b = off + nbytes[i];
        uint64_t s = a > lo ? a : lo, e = b < hi ? b : hi;
        if (s < e)
            memcpy(ptrs[i] + (s - a), buffer + s, e - s);
        off = b;
    }
}

/* Selective restore: verify only the listed chunks (bad[id] is written for them alone), and
 * scatter the payload bytes of each listed chunk -- unless skip_bad is set and the chunk is
 * bad, in which case its tensor ranges keep their old contents.  Returns the number of listed
 * chunks that are bad. */
uint64_t orc_restore_chunks(uint8_t *const *ptrs, const uint64_t *nbytes, uint64_t n_segs,
                            uint64_t chunk_bytes, const uint8_t *buffer, const uint32_t *crcs,
                            const uint64_t *ids, uint64_t n_ids, uint32_t *bad, int skip_bad)
{
    uint64_t payload = total_bytes(nbytes, n_segs), n_bad = 0;
    for (uint64_t k = 0; k < n_ids; k++) {
        uint64_t j = ids[k];
        n_bad += orc_verify_chunks(buffer, crcs, chunk_bytes, bad, j, j + 1);
        if (skip_bad && bad[j])
            continue;
        uint64_t lo = j * chunk_bytes, hi = (j + 1) * chunk_bytes;
        if (hi > payload)
            hi = payload;
        if (lo < hi)
            scatter_range(ptrs, nbytes, n_segs, buffer, lo, hi);
    }
    return n_bad;
}

/* ---- AdamW ----------------------------------------------------------------------------- */

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    uint32_t step;
} orc_adam_hparams;

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16, round to nearest even; a NaN keeps its sign and top payload bits and is
 * forced quiet so that it cannot round to infinity. */
uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

/* IEEE 754 does not fix the sign or payload of a NaN that an operation produces, and processors
 * differ (an x86 subtract hands on its NaN operand, a GPU's add of the negated operand flips the
 * sign).  The snapshot is defined byte for byte and carries CRCs across machines, so the reading
 * taken is: a new master, m or v that is NaN is stored as the one canonical quiet NaN 0x7FC00000,
 * and the 16-bit weight is rounded from that stored value (bf16 0x7FC0, fp16 0x7E00). */
static float canonical_nan(float x)
{
    if (isnan(x)) {
        uint32_t u = 0x7FC00000u;
        memcpy(&x, &u, 4);
    }
    return x;
}

/* Scalars every element shares: derived in double from the fp32 hyper-parameters, then
 * rounded once to fp32. */
typedef struct {
    float decay, b1, omb1, b2, omb2, step_size, bc2s, eps;
} adam_consts;

static adam_consts derive_consts(const orc_adam_hparams *h)
{
    double lr = h->lr, b1 = h->beta1, b2 = h->beta2, wd = h->weight_decay, t = (double)h->step;
    adam_consts k;
    k.decay = (float)(1.0 - lr * wd);
    k.b1 = h->beta1;
    k.omb1 = (float)(1.0 - b1);
    k.b2 = h->beta2;
    k.omb2 = (float)(1.0 - b2);
    k.step_size = (float)(lr / (1.0 - pow(b1, t)));
    k.bc2s = (float)sqrt(1.0 - pow(b2, t));
    k.eps = h->eps;
    return k;
}

/* One decoupled-weight-decay Adam step on n elements, every operation a separately rounded
 * fp32 operation in exactly this order (volatile temporaries forbid contraction or reordering;
 * the file is also built with -ffp-contract=off). */
void orc_adam_f32(uint64_t n, const uint16_t *grad, float *master, float *m, float *v,
                  uint16_t *w16, const orc_adam_hparams *h)
{
    adam_consts k = derive_consts(h);
    for (uint64_t i = 0; i < n; i++) {
        volatile float g = bf16_to_f32(grad[i]);
        volatile float p = master[i] * k.decay;
        volatile float m_a = k.b1 * m[i];
        volatile float m_b = k.omb1 * g;
        volatile float m1 = m_a + m_b;
        volatile float v_a = k.b2 * v[i];
        volatile float v_b = k.omb2 * g;
        volatile float v_c = v_b * g;
        volatile float v1 = v_a + v_c;
        volatile float r = sqrtf(v1);
        volatile float d0 = r / k.bc2s;
        volatile float d = d0 + k.eps;
        volatile float q = m1 / d;
        volatile float u = k.step_size * q;
        volatile float p1 = p - u;
        p1 = canonical_nan(p1);
        master[i] = p1;
        m[i] = canonical_nan(m1);
        v[i] = canonical_nan(v1);
        w16[i] = orc_f32_to_bf16(p1);
    }
}

/* ---- fp16 variant (the paper trains in fp16, section 7.1) ------------------------------------
 * IEEE 754 binary16 decoded by its definition: (-1)^s * 2^(e-15) * (1 + f/1024), subnormals
 * 2^-14 * f/1024; infinities and NaNs keep sign and payload (payload moved to the top bits). */
float orc_f16_to_f32(uint16_t h)
{
    int e = (h >> 10) & 0x1F;
    uint32_t f = h & 0x3FFu;
    float r;
    if (e == 31) {
        uint32_t u = 0x7F800000u | (f << 13);
        memcpy(&r, &u, 4);
    } else if (e == 0) {
        r = (float)ldexp((double)f, -24);
    } else {
        r = (float)ldexp((double)(f + 1024u), e - 25);
    }
    return (h & 0x8000u) ? -r : r;
}

/* binary32 -> binary16, round to nearest even by the definition: the representable neighbours
 * of |x| are multiples of the quantum 2^(max(E, -14) - 10), E = floor(log2 |x|); the nearest
 * multiple is taken (ties to the even one) and anything that rounds to 2^16 or more is
 * infinity.  NaN keeps sign and the top 9 payload bits and is forced quiet. */
uint16_t orc_f32_to_f16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (uint16_t)(sign | 0x7E00u | ((u >> 13) & 0x1FFu));
    double a = fabs((double)x);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
    int ex;
    (void)frexp(a, &ex); /* a = frac * 2^ex, frac in [0.5, 1): E = ex - 1 */
    int E = ex - 1;
    if (E < -14) E = -14;
    double quantum = ldexp(1.0, E - 10);
    double q = nearbyint(a / quantum); /* default rounding mode: to nearest, ties to even */
    double r = q * quantum;
    if (r >= 65536.0) return (uint16_t)(sign | 0x7C00u);
    if (r == 0.0) return sign;
    /* encode r, which is exactly representable */
    (void)frexp(r, &ex);
    E = ex - 1;
    if (E < -14) return (uint16_t)(sign | (uint16_t)ldexp(r, 24)); /* subnormal: f = r * 2^24 */
    uint32_t f = (uint32_t)ldexp(r, 10 - E) - 1024u;
    return (uint16_t)(sign | ((uint32_t)(E + 15) << 10) | f);
}

/* Element-wise conversions of arrays (for tests that sweep every fp16 value). */
void orc_f16_to_f32_array(uint64_t n, const uint16_t *in, float *out)
{
    for (uint64_t i = 0; i < n; i++) out[i] = orc_f16_to_f32(in[i]);
}

void orc_f32_to_f16_array(uint64_t n, const float *in, uint16_t *out)
{
    for (uint64_t i = 0; i < n; i++) out[i] = orc_f32_to_f16(in[i]);
}

/* The Adam step of orc_adam_f32 for fp16 training with a loss scale: the gradient is fp16 and
 * was computed on a loss multiplied by S, so g = float(grad) * inv_scale (inv_scale = 1/S, one
 * rounded fp32 multiplication); the working weights are the fp16 rounding of the new master.
 * *n_nonfinite gets the number of gradient elements that are infinite or NaN (the caller's
 * signal to lower S and to fall back to the previous snapshot); the update itself is applied
 * to every element by the same arithmetic. */
void orc_adam_f32_f16(uint64_t n, const uint16_t *grad, float inv_scale, float *master, float *m,
                      float *v, uint16_t *w16, const orc_adam_hparams *h, uint64_t *n_nonfinite)
{
    adam_consts k = derive_consts(h);
    uint64_t bad = 0;
    for (uint64_t i = 0; i < n; i++) {
        volatile float g_raw = orc_f16_to_f32(grad[i]);
        if (isinf(g_raw) || isnan(g_raw)) bad++;
        volatile float g = g_raw * inv_scale;
        volatile float p = master[i] * k.decay;
        volatile float m_a = k.b1 * m[i];
        volatile float m_b = k.omb1 * g;
        volatile float m1 = m_a + m_b;
        volatile float v_a = k.b2 * v[i];
        volatile float v_b = k.omb2 * g;
        volatile float v_c = v_b * g;
        volatile float v1 = v_a + v_c;
        volatile float r = sqrtf(v1);
        volatile float d0 = r / k.bc2s;
        volatile float d = d0 + k.eps;
        volatile float q = m1 / d;
        volatile float u = k.step_size * q;
        volatile float p1 = p - u;
        p1 = canonical_nan(p1);
        master[i] = p1;
        m[i] = canonical_nan(m1);
        v[i] = canonical_nan(v1);
        w16[i] = orc_f32_to_f16(p1);
    }
    if (n_nonfinite) *n_nonfinite = bad;
}

/* The same step with every quantity in double: the sanity reference for small tensors. */
void orc_adam_f64(uint64_t n, const double *grad, double *master, double *m, double *v,
                  double lr, double beta1, double beta2, double eps, double weight_decay,
                  uint32_t step)
{
    double t = (double)step;
    double step_size = lr / (1.0 - pow(beta1, t));
    double bc2s = sqrt(1.0 - pow(beta2, t));
    for (uint64_t i = 0; i < n; i++) {
        double g = grad[i];
        double p = master[i] * (1.0 - lr * weight_decay);
        double m1 = beta1 * m[i] + (1.0 - beta1) * g;
        double v1 = beta2 * v[i] + (1.0 - beta2) * g * g;
        double d = sqrt(v1) / bc2s + eps;
        master[i] = p - step_size * (m1 / d);
        m[i] = m1;
        v[i] = v1;
    }
}
