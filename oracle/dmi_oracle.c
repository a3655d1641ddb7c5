/*
 * CPU oracle for the capture-and-stage path.  TEST INFRASTRUCTURE ONLY: it is
 * slow on purpose, shares no code with the HIP library, and may be called only
 * from tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * What it computes has a plain definition, written out here with no blocking,
 * fusion or reordering:
 *
 *   - A capture copies a tensor's selected rows, unmodified, into the staging
 *     ring in hook-execution order (paper section 4.2, step 1; section 5,
 *     "Device-to-device kernel"), keeping only retained requests' slices along
 *     the batch dimension (section 4.4, "Policy manager": gather-compact).
 *   - Each capture is published as one record whose fixed 64-byte descriptor
 *     states where the payload is and how long it is (section 4.2, step 2;
 *     section 5).  In this build the descriptor travels in the ring in front of
 *     its payload, followed by the per-request table the paper keeps in its
 *     host-side metadata FIFO (request ids, token ranges; section 4.2).
 *   - Downcasts (bf16 -> fp16, bf16 -> fp8 E4M3FN) are "nearest representable
 *     value, ties to even"; they are found here by searching the target
 *     format's value list, not by bit tricks.
 *   - Per-row summaries (L2 norm, mean, max |x|) are evaluated in float64 from
 *     the exact source values and rounded once to float32.
 *
 * Record layout (little endian, every pad byte zero):
 *   header 64 B : 0 u32 magic 0x32494D44 | 4 u16 version 1 | 6 u16 header_bytes 64
 *                 8 u64 seq | 16 u64 step_id | 24 u32 point_id
 *                 28 u8 src_dtype | 29 u8 out_dtype | 30 u8 summary_mask
 *                 31 u8 flags (1 paged, 2 keep-mask used, 4 explicit row index)
 *                 32 u32 n_reqs | 36 u32 n_rows | 40 u32 row_elems | 44 u32 rank_tag
 *                 48 u64 record_bytes | 56 u64 payload_bytes
 *   req table   : n_reqs x { u32 req_id, u32 tok_start, u32 tok_step, u32 n_rows_r }, pad to 64
 *   payload     : n_rows x row_elems x sizeof(out_dtype), request-major then
 *                 token-ascending, tightly packed, pad to 64 (absent if out_dtype NONE)
 *   summaries   : for each set bit of summary_mask, ascending (1 L2, 2 mean,
 *                 4 absmax): f32[n_rows], each array padded to 64
 *
 * What pins this file to something other than itself (tests/test_oracle_*.py, no GPU):
 *   - gathers: the all-rows case equals a memcpy of the tensor; ragged selections equal
 *     torch.index_select on the same bytes; a paged cache whose elements encode
 *     (block, slot, head, dim) decodes to exactly the rows asked for, and an identity
 *     block table reduces the paged gather to the dense one;
 *   - bf16 -> fp16: all 65,536 inputs against torch's CPU cast (a library routine), and
 *     closed-form values (overflow to inf, ties, subnormals, NaN payload);
 *   - bf16 -> fp8: all inputs with |x| <= 464 against torch's CPU float8_e4m3fn cast, all
 *     65,536 against a separate linear scan over the 254 finite codes, and closed-form
 *     values (448, 464, 1.0, 2^-9, 2^-10, -0, saturation, NaN);
 *   - summaries: constant, one-hot and alternating rows (closed forms), numpy float64 as a
 *     second route, NaN / inf rows;
 *   - layout: an independent decoder (decode.py) recomputes every size and checks every
 *     pad byte over random shapes.
 * Parity unpinned: the record layout itself.  The paper prints no byte values (it speaks of
 * a 64-byte descriptor with offset, length and ready flag); the layout above is this
 * build's, checked for self-consistency only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { DT_NONE = 0, DT_BF16 = 1, DT_FP16 = 2, DT_FP32 = 3, DT_FP8 = 4 };
enum { SUM_L2 = 1, SUM_MEAN = 2, SUM_ABSMAX = 4 };
enum { FLAG_PAGED = 1, FLAG_MASK = 2, FLAG_INDEX = 4 };

typedef struct {
    uint32_t req_id, row_base, tok_start, tok_count, tok_step;
} orc_req_t;

typedef struct {
    const void *data;
    uint32_t dtype;
    int64_t n_rows;      /* T */
    int64_t row_elems;   /* E */
    int64_t row_stride;  /* elements between consecutive rows */
} orc_dense_t;

typedef struct {
    const void *base;
    uint32_t dtype;
    int64_t block_stride, slot_stride, head_stride; /* elements */
    uint32_t block_size, n_heads, head_dim;
    const int32_t *block_table;
    int64_t block_table_stride;                     /* entries per sequence */
    uint32_t n_heads_sel;
    uint32_t heads_sel[8];
} orc_paged_t;

/* ------------------------------------------------------------------ values */

static double f32_bits_value(uint32_t u)
{
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* bf16 is the upper half of an IEEE binary32 */
double orc_bf16_value(uint16_t b) { return f32_bits_value((uint32_t)b << 16); }

/* IEEE binary16 code -> value, from the format definition */
double orc_fp16_value(uint16_t h)
{
    int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -24);            /* 2^-14 * m/1024 */
    else v = ldexp(1.0 + m / 1024.0, e - 15);
    return s ? -v : v;
}

/* OCP FP8 E4M3FN code -> value: bias 7, no infinities, S.1111.111 is NaN */
double orc_fp8_value(uint8_t c)
{
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) v = NAN;
    else if (e == 0) v = ldexp((double)m, -9);             /* 2^-6 * m/8 */
    else v = ldexp(1.0 + m / 8.0, e - 7);
    return s ? -v : v;
}

/*
 * Nearest code among magnitudes mag(0) < mag(1) < ... < mag(top), ties to the
 * even code (codes are sign-magnitude, so an even code has an even mantissa).
 */
static uint32_t nearest_code(double ax, uint32_t top, double (*mag)(uint32_t))
{
    uint32_t lo = 0, hi = top; /* invariant: mag(lo) <= ax, or lo == 0 */
    if (ax >= mag(top)) return top;
    while (hi - lo > 1) {
        uint32_t mid = lo + (hi - lo) / 2;
        if (mag(mid) <= ax) lo = mid; else hi = mid;
    }
    {
        double dl = ax - mag(lo), dh = mag(hi) - ax;
        if (dl < dh) return lo;
        if (dh < dl) return hi;
        return (lo & 1) ? hi : lo;
    }
}

static double fp8_mag(uint32_t c) { return orc_fp8_value((uint8_t)c); }

/* top code 0x7C00 stands for 2^16, the value the next binade would start at:
 * rounding as if the exponent range were unbounded, then overflow -> inf. */
static double fp16_mag(uint32_t c) { return c == 0x7C00 ? 65536.0 : orc_fp16_value((uint16_t)c); }

/* bf16 -> fp8 E4M3FN: nearest finite value, ties to even, saturating (values
 * beyond the largest finite 448, infinities included, give +-448); NaN -> NaN. */
uint8_t orc_bf16_to_fp8(uint16_t b)
{
    uint8_t s = (uint8_t)((b >> 15) << 7);
    double x = orc_bf16_value(b);
    if (isnan(x)) return s | 0x7F;
    return s | (uint8_t)nearest_code(fabs(x), 0x7E, fp8_mag);
}

/* bf16 -> fp16: IEEE round-to-nearest-even, overflow to infinity, gradual
 * underflow; NaN -> quiet NaN 0x7E00 with the sign kept. */
uint16_t orc_bf16_to_fp16(uint16_t b)
{
    uint16_t s = (uint16_t)((b >> 15) << 15);
    double x = orc_bf16_value(b);
    if (isnan(x)) return s | 0x7E00;
    if (isinf(x)) return s | 0x7C00;
    return s | (uint16_t)nearest_code(fabs(x), 0x7C00, fp16_mag);
}

/* The two conversions above evaluated once for all 65,536 bf16 inputs and
 * remembered (a memo of the definition, so that large test cases finish). */
static uint8_t fp8_memo[65536];
static uint16_t fp16_memo[65536];
static int memo_ready;

static void build_memo(void)
{
    for (uint32_t b = 0; b < 65536; b++) {
        fp8_memo[b] = orc_bf16_to_fp8((uint16_t)b);
        fp16_memo[b] = orc_bf16_to_fp16((uint16_t)b);
    }
    memo_ready = 1;
}

static uint32_t dtype_size(uint32_t dt)
{
    switch (dt) {
    case DT_BF16: case DT_FP16: return 2;
    case DT_FP32: return 4;
    case DT_FP8: return 1;
    default: return 0;
    }
}
uint32_t orc_dtype_size(uint32_t dt) { return dtype_size(dt); }

static uint64_t pad64(uint64_t n) { return (n + 63) / 64 * 64; }

static int popcount3(uint32_t m) { return (int)((m & 1) + ((m >> 1) & 1) + ((m >> 2) & 1)); }

uint64_t orc_record_bytes(uint32_t n_reqs, uint64_t n_rows, uint32_t row_elems,
                          uint32_t out_dtype, uint32_t summary_mask)
{
    uint64_t b = 64;
    b += pad64((uint64_t)n_reqs * 16);
    b += pad64(n_rows * row_elems * dtype_size(out_dtype));
    b += (uint64_t)popcount3(summary_mask) * pad64(n_rows * 4);
    return b;
}

/* source element -> exact value */
static double src_value(const void *p, uint32_t dt)
{
    if (dt == DT_BF16) { uint16_t b; memcpy(&b, p, 2); return orc_bf16_value(b); }
    if (dt == DT_FP16) { uint16_t h; memcpy(&h, p, 2); return orc_fp16_value(h); }
    { float f; memcpy(&f, p, 4); return (double)f; }
}

static void put_u16(uint8_t *p, uint16_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put_u32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void put_u64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void put_f32(uint8_t *p, float f) { uint32_t u; memcpy(&u, &f, 4); put_u32(p, u); }

/* one source element -> its bytes in the payload */
static void emit_elem(uint8_t *dst, const uint8_t *src, uint32_t src_dt, uint32_t out_dt)
{
    if (out_dt == src_dt) {
        memcpy(dst, src, dtype_size(src_dt));
    } else if (src_dt == DT_BF16 && out_dt == DT_FP16) {
        uint16_t b; memcpy(&b, src, 2);
        put_u16(dst, fp16_memo[b]);
    } else if (src_dt == DT_BF16 && out_dt == DT_FP8) {
        uint16_t b; memcpy(&b, src, 2);
        dst[0] = fp8_memo[b];
    }
}

int orc_transform_supported(uint32_t src_dt, uint32_t out_dt)
{
    if (src_dt != DT_BF16 && src_dt != DT_FP16 && src_dt != DT_FP32) return 0;
    if (out_dt == DT_NONE || out_dt == src_dt) return 1;
    return src_dt == DT_BF16 && (out_dt == DT_FP16 || out_dt == DT_FP8);
}

/*
 * Row source abstraction: a row is n_seg segments of seg_elems contiguous
 * elements.  Dense: one segment, the row.  Paged: one segment per selected head.
 */
typedef struct {
    const orc_dense_t *d;
    const orc_paged_t *p;
} row_src_t;

static const uint8_t *segment_ptr(const row_src_t *s, const orc_req_t *rq, int64_t row_or_tok,
                                  uint32_t seg)
{
    if (s->d) {
        uint32_t es = dtype_size(s->d->dtype);
        return (const uint8_t *)s->d->data + row_or_tok * s->d->row_stride * es;
    } else {
        const orc_paged_t *p = s->p;
        uint32_t es = dtype_size(p->dtype);
        int64_t t = row_or_tok;
        int64_t blk = p->block_table[(int64_t)rq->row_base * p->block_table_stride + t / p->block_size];
        int64_t off = blk * p->block_stride + (t % p->block_size) * p->slot_stride +
                      (int64_t)p->heads_sel[seg] * p->head_stride;
        return (const uint8_t *)p->base + off * es;
    }
}

/*
 * Build one record into out[0 .. return value).  Returns the record size, or
 * -1 for an unsupported transform, -2 if out_cap is too small, -3 if a
 * selection leaves the tensor.
 */
static int64_t build_record(uint8_t *out, uint64_t out_cap, uint64_t seq, uint64_t step_id,
                            uint32_t point_id, uint32_t rank_tag, const row_src_t *src,
                            const orc_req_t *reqs, uint32_t n_reqs, const uint8_t *keep_mask,
                            const int32_t *row_index, uint32_t out_dtype, uint32_t summary_mask)
{
    uint32_t src_dt = src->d ? src->d->dtype : src->p->dtype;
    uint32_t n_seg = src->d ? 1 : src->p->n_heads_sel;
    uint32_t seg_elems = src->d ? (uint32_t)src->d->row_elems : src->p->head_dim;
    uint32_t row_elems = n_seg * seg_elems;
    uint32_t es_in = dtype_size(src_dt), es_out = dtype_size(out_dtype);
    uint64_t n_rows = 0;
    uint8_t flags = 0;

    if (!orc_transform_supported(src_dt, out_dtype) || (summary_mask & ~7u)) return -1;
    if (!memo_ready) build_memo();
    if (src->p && row_index) return -1;
    for (uint32_t r = 0; r < n_reqs; r++)
        if (!keep_mask || keep_mask[r]) n_rows += reqs[r].tok_count;
    if (src->p) flags |= FLAG_PAGED;
    if (keep_mask) flags |= FLAG_MASK;
    if (row_index) flags |= FLAG_INDEX;

    uint64_t table_bytes = pad64((uint64_t)n_reqs * 16);
    uint64_t payload_bytes = n_rows * row_elems * es_out;
    uint64_t sum_bytes = pad64(n_rows * 4);
    uint64_t total = orc_record_bytes(n_reqs, n_rows, row_elems, out_dtype, summary_mask);
    if (total > out_cap) return -2;
    memset(out, 0, total);

    /* header */
    put_u32(out + 0, 0x32494D44u);
    put_u16(out + 4, 1);
    put_u16(out + 6, 64);
    put_u64(out + 8, seq);
    put_u64(out + 16, step_id);
    put_u32(out + 24, point_id);
    out[28] = (uint8_t)src_dt;
    out[29] = (uint8_t)out_dtype;
    out[30] = (uint8_t)summary_mask;
    out[31] = flags;
    put_u32(out + 32, n_reqs);
    put_u32(out + 36, (uint32_t)n_rows);
    put_u32(out + 40, row_elems);
    put_u32(out + 44, rank_tag);
    put_u64(out + 48, total);
    put_u64(out + 56, payload_bytes);

    /* request table */
    for (uint32_t r = 0; r < n_reqs; r++) {
        uint8_t *e = out + 64 + (uint64_t)r * 16;
        int kept = !keep_mask || keep_mask[r];
        put_u32(e + 0, reqs[r].req_id);
        put_u32(e + 4, reqs[r].tok_start);
        put_u32(e + 8, reqs[r].tok_step);
        put_u32(e + 12, kept ? reqs[r].tok_count : 0);
    }

    uint8_t *payload = out + 64 + table_bytes;
    uint8_t *sums = payload + pad64(payload_bytes);
    uint8_t *sum_l2 = NULL, *sum_mean = NULL, *sum_amax = NULL;
    {
        uint8_t *p = sums;
        if (summary_mask & SUM_L2) { sum_l2 = p; p += sum_bytes; }
        if (summary_mask & SUM_MEAN) { sum_mean = p; p += sum_bytes; }
        if (summary_mask & SUM_ABSMAX) { sum_amax = p; p += sum_bytes; }
    }

    uint64_t g = 0;          /* output row */
    uint64_t listed = 0;     /* position in row_index: advances over masked-out requests too */
    for (uint32_t r = 0; r < n_reqs; r++) {
        const orc_req_t *rq = &reqs[r];
        int kept = !keep_mask || keep_mask[r];
        for (uint32_t j = 0; j < rq->tok_count; j++, listed++) {
            if (!kept) continue;
            int64_t where;
            if (src->d) {
                where = row_index ? (int64_t)row_index[listed]
                                  : (int64_t)rq->row_base + rq->tok_start + (int64_t)j * rq->tok_step;
                if (where < 0 || where >= src->d->n_rows) return -3;
            } else {
                where = (int64_t)rq->tok_start + (int64_t)j * rq->tok_step; /* logical token */
            }
            double sumsq = 0.0, sum = 0.0, amax = 0.0;
            int has_nan = 0;
            for (uint32_t sg = 0; sg < n_seg; sg++) {
                const uint8_t *sp = segment_ptr(src, rq, where, sg);
                for (uint32_t c = 0; c < seg_elems; c++) {
                    const uint8_t *ep = sp + (uint64_t)c * es_in;
                    if (es_out)
                        emit_elem(payload + (g * row_elems + (uint64_t)sg * seg_elems + c) * es_out,
                                  ep, src_dt, out_dtype);
                    if (summary_mask) {
                        double v = src_value(ep, src_dt);
                        sumsq += v * v;
                        sum += v;
                        if (isnan(v)) has_nan = 1;
                        else if (fabs(v) > amax) amax = fabs(v);
                    }
                }
            }
            if (sum_l2) put_f32(sum_l2 + g * 4, (float)sqrt(sumsq));
            if (sum_mean) put_f32(sum_mean + g * 4, (float)(sum / (double)row_elems));
            if (sum_amax) put_f32(sum_amax + g * 4, has_nan ? NAN : (float)amax);
            g++;
        }
    }
    return (int64_t)total;
}

int64_t orc_build_dense(uint8_t *out, uint64_t out_cap, uint64_t seq, uint64_t step_id,
                        uint32_t point_id, uint32_t rank_tag, const orc_dense_t *t,
                        const orc_req_t *reqs, uint32_t n_reqs, const uint8_t *keep_mask,
                        const int32_t *row_index, uint32_t out_dtype, uint32_t summary_mask)
{
    row_src_t s = { t, NULL };
    return build_record(out, out_cap, seq, step_id, point_id, rank_tag, &s, reqs, n_reqs,
                        keep_mask, row_index, out_dtype, summary_mask);
}

int64_t orc_build_paged(uint8_t *out, uint64_t out_cap, uint64_t seq, uint64_t step_id,
                        uint32_t point_id, uint32_t rank_tag, const orc_paged_t *kv,
                        const orc_req_t *reqs, uint32_t n_reqs, const uint8_t *keep_mask,
                        uint32_t out_dtype, uint32_t summary_mask)
{
    row_src_t s = { NULL, kv };
    return build_record(out, out_cap, seq, step_id, point_id, rank_tag, &s, reqs, n_reqs,
                        keep_mask, NULL, out_dtype, summary_mask);
}
