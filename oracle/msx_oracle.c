/*
 * CPU oracle for the emulated-rank collective hot path (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the slow, single-threaded, obviously-correct statement of what each
 * collective computes.  It is used only by the tests, by the smoke check and by the
 * benchmark's CPU-baseline leg; the product library never links, loads or calls it,
 * and it shares no code, header, table or helper with the HIP implementation.
 *
 * Everything here is a plain definition written out:
 *   - AllReduce / ReduceScatter / AllGather follow the problem statement in the paper's
 *     "Collective Communications" background section (AllReduce sums the inputs of all
 *     ranks and every rank gets the result; ReduceScatter sums and hands each rank an
 *     equal share; AllGather concatenates the shares on every rank).
 *   - The LL unit follows the MemoryChannel "Protocols" paragraph: a data word and a
 *     flag travel in one store; a reader accepts the data only when the flag matches.
 *   - The token dispatch follows the expert-parallel setting the paper evaluates
 *     (hidden 7168, top-8 of 256 experts); the paper does not define the packing order,
 *     so the order used here (source rank ascending, then token ascending, one copy per
 *     distinct destination rank) is this build's reading.
 *
 * Readings of points the paper leaves open (reduction order, accumulator width,
 * rounding) are: fp32 accumulator, ranks added in order 0,1,...,N-1 starting from rank
 * 0's value, one round-to-nearest-even conversion to bf16 at the end.
 *
 * Every function is pinned by tests that do not re-use its own formula (closed forms,
 * exact integer sums, a library column-sum, permutation identities, brute force).
 * Performance figures have no pin: the paper prints no number for emulated ranks.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ---------- bf16 <-> fp32 (IEEE binary32 truncated to its top 16 bits) ---------- */

float orc_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest, ties-to-even; NaN stays NaN (quiet bit forced, sign kept) */
uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

void orc_bf16_to_f32_buf(const uint16_t *in, float *out, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        out[i] = orc_bf16_to_f32(in[i]);
}

void orc_f32_to_bf16_buf(const float *in, uint16_t *out, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        out[i] = orc_f32_to_bf16(in[i]);
}

/* ---------- AllReduce (sum) ---------- */

/* in: [n][count] rank-major.  out: [count] (the value every rank must hold). */
void orc_allreduce_f32(const float *in, float *out, int n, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        float acc = in[i];
        for (int r = 1; r < n; ++r)
            acc += in[(size_t)r * count + i];
        out[i] = acc;
    }
}

/* exact integer sum of integer-valued fp32 inputs (order-free check for config 1).
 * returns 0 if every input was an integer of magnitude < 2^31, else 1. */
int orc_allreduce_f32_as_i64(const float *in, int64_t *out, int n, size_t count)
{
    int bad = 0;
    for (size_t i = 0; i < count; ++i) {
        int64_t acc = 0;
        for (int r = 0; r < n; ++r) {
            float v = in[(size_t)r * count + i];
            if (!(v > -2147483648.0f && v < 2147483648.0f) || (float)(int64_t)v != v)
                bad = 1;
            else
                acc += (int64_t)v;
        }
        out[i] = acc;
    }
    return bad;
}

/* in: [n][count] bf16 bit patterns.  out: [count] bf16.  ref64 (nullable): [count]
 * the same sum accumulated in double, unrounded. */
void orc_allreduce_bf16(const uint16_t *in, uint16_t *out, double *ref64, int n, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        float acc = orc_bf16_to_f32(in[i]);
        double wide = (double)acc;
        for (int r = 1; r < n; ++r) {
            float v = orc_bf16_to_f32(in[(size_t)r * count + i]);
            acc += v;
            wide += (double)v;
        }
        out[i] = orc_f32_to_bf16(acc);
        if (ref64)
            ref64[i] = wide;
    }
}

/* AllReduce fused with a residual add, as seen by ONE rank whose residual is res:
 * out[i] = bf16( (sum over ranks in fp32) + fp32(res[i]) ), a single rounding. */
void orc_allreduce_residual_bf16(const uint16_t *in, const uint16_t *res, uint16_t *out,
                                 double *ref64, int n, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        float acc = orc_bf16_to_f32(in[i]);
        double wide = (double)acc;
        for (int r = 1; r < n; ++r) {
            float v = orc_bf16_to_f32(in[(size_t)r * count + i]);
            acc += v;
            wide += (double)v;
        }
        float rv = orc_bf16_to_f32(res[i]);
        acc += rv;
        wide += (double)rv;
        out[i] = orc_f32_to_bf16(acc);
        if (ref64)
            ref64[i] = wide;
    }
}

void orc_allreduce_residual_f32(const float *in, const float *res, float *out, int n, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        float acc = in[i];
        for (int r = 1; r < n; ++r)
            acc += in[(size_t)r * count + i];
        acc += res[i];
        out[i] = acc;
    }
}

/* ---------- fp16 (IEEE binary16) and the other reduction operators ----------
 * The paper's DSL carries a ReduceOp and the NCCL-style API more element types than the two the
 * configurations use; these cover fp16 and max / min.  Sum is taken in fp32 in rank order and
 * rounded once; max / min compare in fp32 in rank order and keep the earlier value unless the
 * later one is strictly greater / smaller (so a NaN in a later rank never replaces a number, and
 * a NaN in rank 0 stays). */

float orc_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31, e = (h >> 10) & 31u, m = h & 1023u, u;
    if (e == 31)
        u = sign | 0x7f800000u | (m << 13);
    else if (e == 0) {
        if (m == 0)
            u = sign;
        else {                                   /* subnormal: normalise */
            int shift = 0;
            while (!(m & 1024u)) { m <<= 1; ++shift; }
            u = sign | ((uint32_t)(113 - shift) << 23) | ((m & 1023u) << 13);
        }
    } else
        u = sign | ((e + 112u) << 23) | (m << 13);
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round to nearest even; overflow to infinity; NaN stays NaN (quiet) */
uint16_t orc_f32_to_f16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u)
        return (uint16_t)(sign | 0x7e00u | ((a >> 13) & 0x3ffu));
    if (a >= 0x477ff000u)                        /* rounds to 65536 or more: infinity */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x38800000u) {                       /* below 2^-14: fp16 subnormal, multiples of 2^-24 */
        if (a < 0x33000000u)                     /* below 2^-25: rounds to zero (2^-25 itself ties to even = 0) */
            return (uint16_t)(sign | (a > 0x33000000u ? 1u : 0u));
        uint32_t e = a >> 23, m = (a & 0x7fffffu) | 0x800000u;
        uint32_t shift = 126u - e;               /* result = m >> shift, in units of 2^-24 */
        uint32_t q = m >> shift, rem = m & ((1u << shift) - 1u), half = 1u << (shift - 1);
        if (rem > half || (rem == half && (q & 1u)))
            ++q;
        return (uint16_t)(sign | q);
    }
    uint32_t r = a + 0xfffu + ((a >> 13) & 1u);
    return (uint16_t)(sign | (uint16_t)((r - 0x38000000u) >> 13));
}

static float orc_load_elem(const void *p, size_t i, int dtype)
{
    if (dtype == 0) return ((const float *)p)[i];
    if (dtype == 1) return orc_bf16_to_f32(((const uint16_t *)p)[i]);
    return orc_f16_to_f32(((const uint16_t *)p)[i]);
}

static void orc_store_elem(void *p, size_t i, int dtype, float v)
{
    if (dtype == 0) ((float *)p)[i] = v;
    else if (dtype == 1) ((uint16_t *)p)[i] = orc_f32_to_bf16(v);
    else ((uint16_t *)p)[i] = orc_f32_to_f16(v);
}

/* dtype: 0 fp32, 1 bf16, 2 fp16, 3 int32.  op: 0 sum, 1 max, 2 min.  in: [n][count] -> out: [count].
 * int32: the sum is taken modulo 2^32 (two's complement wrap-around, no trap), max / min are signed. */
void orc_allreduce_any(const void *in, void *out, int n, size_t count, int dtype, int op)
{
    if (dtype == 3) {
        const int32_t *x = (const int32_t *)in;
        int32_t *o = (int32_t *)out;
        for (size_t i = 0; i < count; ++i) {
            int32_t acc = x[i];
            for (int r = 1; r < n; ++r) {
                int32_t v = x[(size_t)r * count + i];
                if (op == 0) acc = (int32_t)((uint32_t)acc + (uint32_t)v);
                else if (op == 1) acc = v > acc ? v : acc;
                else acc = v < acc ? v : acc;
            }
            o[i] = acc;
        }
        return;
    }
    size_t esz = dtype == 0 ? 4 : 2;
    for (size_t i = 0; i < count; ++i) {
        float acc = orc_load_elem(in, i, dtype);
        for (int r = 1; r < n; ++r) {
            float v = orc_load_elem((const char *)in + (size_t)r * count * esz, i, dtype);
            if (op == 0) acc += v;
            else if (op == 1) acc = v > acc ? v : acc;
            else acc = v < acc ? v : acc;
        }
        orc_store_elem(out, i, dtype, acc);
    }
}

/* ---------- ring order (two-phase ring AllReduce, Collectives Library section, 2PR) ----------
 * The buffer is cut into n equal chunks; chunk k starts at rank k and travels k -> k+1 -> ... ->
 * k-1 (mod n); every rank on the way adds its own values in fp32 and passes the partial sum on
 * in the element type, so the partial is rounded to that type at every hop.  The all-gather
 * phase then copies the finished chunk to everybody.  count % n == 0.  out: [count]. */
void orc_allreduce_ring_bf16(const uint16_t *in, uint16_t *out, int n, size_t count)
{
    size_t c = count / (size_t)n;
    for (int k = 0; k < n; ++k)
        for (size_t i = (size_t)k * c; i < (size_t)(k + 1) * c; ++i) {
            uint16_t part = in[(size_t)k * count + i];
            for (int h = 1; h < n; ++h) {
                int r = (k + h) % n;
                float acc = orc_bf16_to_f32(part) + orc_bf16_to_f32(in[(size_t)r * count + i]);
                part = orc_f32_to_bf16(acc);
            }
            out[i] = part;
        }
}

void orc_allreduce_ring_f32(const float *in, float *out, int n, size_t count)
{
    size_t c = count / (size_t)n;
    for (int k = 0; k < n; ++k)
        for (size_t i = (size_t)k * c; i < (size_t)(k + 1) * c; ++i) {
            float part = in[(size_t)k * count + i];
            for (int h = 1; h < n; ++h)
                part = part + in[(size_t)((k + h) % n) * count + i];
            out[i] = part;
        }
}

/* ---------- ReduceScatter (sum): rank r receives the sum of everybody's share r ---------- */

/* in: [n][count], count divisible by n.  out: [n][count/n]; row r = rank r's result. */
void orc_reducescatter_f32(const float *in, float *out, int n, size_t count)
{
    size_t c = count / (size_t)n;
    for (int r = 0; r < n; ++r)
        for (size_t k = 0; k < c; ++k) {
            float acc = in[(size_t)r * c + k];
            for (int j = 1; j < n; ++j)
                acc += in[(size_t)j * count + (size_t)r * c + k];
            out[(size_t)r * c + k] = acc;
        }
}

void orc_reducescatter_bf16(const uint16_t *in, uint16_t *out, int n, size_t count)
{
    size_t c = count / (size_t)n;
    for (int r = 0; r < n; ++r)
        for (size_t k = 0; k < c; ++k) {
            float acc = orc_bf16_to_f32(in[(size_t)r * c + k]);
            for (int j = 1; j < n; ++j)
                acc += orc_bf16_to_f32(in[(size_t)j * count + (size_t)r * c + k]);
            out[(size_t)r * c + k] = orc_f32_to_bf16(acc);
        }
}

/* ---------- AllGather / equal AllToAll: pure byte movement ---------- */

/* in: [n][cbytes] (rank j's contribution).  out: [n][n*cbytes]; every row is the
 * concatenation of the contributions in rank order. */
void orc_allgather(const uint8_t *in, uint8_t *out, int n, size_t cbytes)
{
    for (int r = 0; r < n; ++r)
        for (int j = 0; j < n; ++j)
            for (size_t b = 0; b < cbytes; ++b)
                out[((size_t)r * n + j) * cbytes + b] = in[(size_t)j * cbytes + b];
}

/* in: [n][n*cbytes]; slot d of row s is what s sends to d.  out: [n][n*cbytes];
 * slot s of row d is what d received from s. */
void orc_alltoall(const uint8_t *in, uint8_t *out, int n, size_t cbytes)
{
    for (int d = 0; d < n; ++d)
        for (int s = 0; s < n; ++s)
            for (size_t b = 0; b < cbytes; ++b)
                out[((size_t)d * n + s) * cbytes + b] = in[((size_t)s * n + d) * cbytes + b];
}

/* ---------- LL units ---------- */

/* one 8-byte unit: data word in the low half, flag in the high half (little endian:
 * bytes 0-3 data, bytes 4-7 flag, i.e. the flag is the last element of the unit). */
uint64_t orc_ll_encode(uint32_t data, uint32_t flag)
{
    return ((uint64_t)flag << 32) | (uint64_t)data;
}

/* returns 1 and stores the data word if the unit carries the expected flag, else 0 */
int orc_ll_decode(uint64_t unit, uint32_t expect, uint32_t *data)
{
    if ((uint32_t)(unit >> 32) != expect)
        return 0;
    *data = (uint32_t)unit;
    return 1;
}

/* Encode nbytes of payload into 16-byte packets (two units each).  The payload is
 * taken as little-endian 32-bit words; a final partial word and a missing second word
 * are padded with zero data.  units must hold 2*ceil(nbytes/8) entries.
 * Returns the number of units written. */
size_t orc_ll_encode_buf(const uint8_t *payload, size_t nbytes, uint32_t flag, uint64_t *units)
{
    size_t npackets = (nbytes + 7) / 8;
    for (size_t p = 0; p < npackets; ++p)
        for (int h = 0; h < 2; ++h) {
            uint32_t w = 0;
            for (int b = 0; b < 4; ++b) {
                size_t pos = p * 8 + (size_t)h * 4 + (size_t)b;
                if (pos < nbytes)
                    w |= (uint32_t)payload[pos] << (8 * b);
            }
            units[2 * p + (size_t)h] = orc_ll_encode(w, flag);
        }
    return 2 * npackets;
}

/* Decode: returns 1 and fills payload[0..nbytes) iff EVERY unit carries the flag. */
int orc_ll_decode_buf(const uint64_t *units, size_t nbytes, uint32_t flag, uint8_t *payload)
{
    size_t npackets = (nbytes + 7) / 8;
    for (size_t u = 0; u < 2 * npackets; ++u) {
        uint32_t w;
        if (!orc_ll_decode(units[u], flag, &w))
            return 0;
        for (int b = 0; b < 4; ++b) {
            size_t pos = u * 4 + (size_t)b;
            if (pos < nbytes)
                payload[pos] = (uint8_t)(w >> (8 * b));
        }
    }
    return 1;
}

/* ---------- token-routed dispatch ---------- */

/*
 * tokens   : [n][T][row_bytes]   source rows
 * topk     : [n][T][K]           expert ids in [0, n_experts); experts are split evenly,
 *                                expert e lives on rank e / (n_experts / n)
 * recv     : [n][cap][row_bytes] destination buffers (cap rows each); rows beyond the
 *                                received count are left untouched
 * recv_src : [n][cap]            s*T + t of each received row (nullable)
 * counts   : [n dst][n src]      rows destination d received from source s
 * Returns 0, or -1 if some destination would overflow cap (nothing more is written to
 * that destination), or -2 on an out-of-range expert id.
 * A token goes ONCE to each distinct destination rank among its K experts.  Order in a
 * destination buffer: by source rank ascending, then by token index ascending.
 */
int orc_moe_dispatch(const uint8_t *tokens, const int32_t *topk, int n, int T, int K,
                     int n_experts, size_t row_bytes, uint8_t *recv, int32_t *recv_src,
                     int32_t *counts, size_t cap)
{
    int per = n_experts / n;
    int rc = 0;
    for (int d = 0; d < n; ++d) {
        size_t fill = 0;
        for (int s = 0; s < n; ++s) {
            int32_t got = 0;
            for (int t = 0; t < T; ++t) {
                int hit = 0;
                for (int k = 0; k < K; ++k) {
                    int32_t e = topk[((size_t)s * T + t) * K + k];
                    if (e < 0 || e >= n_experts)
                        return -2;
                    if (e / per == d)
                        hit = 1;
                }
                if (!hit)
                    continue;
                if (fill >= cap) {
                    rc = -1;
                    continue;
                }
                memcpy(recv + ((size_t)d * cap + fill) * row_bytes,
                       tokens + ((size_t)s * T + t) * row_bytes, row_bytes);
                if (recv_src)
                    recv_src[(size_t)d * cap + fill] = (int32_t)(s * T + t);
                ++fill;
                ++got;
            }
            counts[d * n + s] = got;
        }
    }
    return rc;
}

/* ---------- FP8 (OCP E4M3: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits; largest finite
 * value 448 = 0x7E, 0x7F / 0xFF are NaN, there is no infinity) ---------- */

float orc_e4m3_to_f32(uint8_t b)
{
    int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
    float v;
    if (e == 15 && m == 7) {
        uint32_t q = 0x7fc00000u | ((uint32_t)sign << 31);
        memcpy(&v, &q, 4);
        return v;
    }
    if (e == 0)
        v = (float)m / 8.0f / 64.0f;                 /* subnormal: m/8 * 2^-6 */
    else {
        v = 1.0f + (float)m / 8.0f;
        for (int i = e; i < 7; ++i) v *= 0.5f;
        for (int i = 7; i < e; ++i) v *= 2.0f;
    }
    return sign ? -v : v;
}

/* nearest representable value, ties to the even code, magnitudes beyond 448 saturate to 448,
 * NaN -> 0x7F.  Written as a search over the 127 finite magnitudes so that it shares nothing
 * with a bit-twiddling encoder. */
uint8_t orc_f32_to_e4m3(float f)
{
    if (f != f)
        return 0x7f;
    uint8_t sign = 0;
    if (f < 0.0f || (f == 0.0f && 1.0f / f < 0.0f)) {
        sign = 0x80;
        f = -f;
    }
    if (f >= 448.0f)
        return (uint8_t)(sign | 0x7e);
    int best = 0;
    for (int code = 0; code < 0x7f; ++code) {        /* magnitudes ascend with the code */
        float lo = orc_e4m3_to_f32((uint8_t)code), hi = orc_e4m3_to_f32((uint8_t)(code + 1));
        if (code + 1 == 0x7f)
            hi = 512.0f;                             /* the value the next code would have had */
        if (f >= lo && f <= hi) {
            double dl = (double)f - (double)lo, dh = (double)hi - (double)f;
            if (dl < dh) best = code;
            else if (dh < dl) best = code + 1;
            else best = (code & 1) ? code + 1 : code;
            break;
        }
    }
    if (best >= 0x7f)
        best = 0x7e;
    return (uint8_t)(sign | best);
}

/* Row-wise quantisation in groups of 128 elements (the 1x128 tile scaling of the DeepSeek-V3
 * setting the paper's expert-parallel experiment uses): amax = max(|x|, 1e-4) over the group,
 * inv = 448 / amax, q = e4m3(x * inv), scale = amax / 448, all in fp32.
 *   x : [rows][H] bf16 bits, H % 128 == 0     q : [rows][H] bytes     scales : [rows][H/128] */
void orc_fp8_quantize_rows(const uint16_t *x, uint8_t *q, float *scales, size_t rows, size_t H)
{
    size_t groups = H / 128;
    for (size_t r = 0; r < rows; ++r)
        for (size_t g = 0; g < groups; ++g) {
            const uint16_t *px = x + r * H + g * 128;
            float amax = 1e-4f;
            for (int i = 0; i < 128; ++i) {
                float v = orc_bf16_to_f32(px[i]);
                if (v < 0.0f) v = -v;
                if (v > amax) amax = v;              /* NaN never wins the comparison */
            }
            float inv = 448.0f / amax;
            scales[r * groups + g] = amax / 448.0f;
            for (int i = 0; i < 128; ++i)
                q[r * H + g * 128 + i] = orc_f32_to_e4m3(orc_bf16_to_f32(px[i]) * inv);
        }
}

/*
 * Combine: the way back of the dispatch.  y[d] holds one processed row for every row that
 * destination d received, in the order the dispatch delivered them.  Every source token
 * gets the sum of its rows over the destination ranks it was sent to, added in fp32 in
 * ascending rank order starting from the first one, rounded once to bf16.
 *   y   : [n][cap][H] bf16 bits        out : [n][T][H] bf16 bits
 * The paper names the operation (dispatch and combine of its expert-parallel experiment)
 * but not the arithmetic; plain unweighted sum in rank order is this build's reading.
 * Returns 0, -1 if a destination would overflow cap, -2 on a bad expert id.
 */
int orc_moe_combine_bf16(const uint16_t *y, const int32_t *topk, int n, int T, int K, int n_experts,
                         size_t H, size_t cap, uint16_t *out, float *acc /* scratch [n*T*H] */,
                         uint8_t *seen /* scratch [n*T] */)
{
    int per = n_experts / n;
    memset(seen, 0, (size_t)n * T);
    for (int d = 0; d < n; ++d) {
        size_t fill = 0;
        for (int s = 0; s < n; ++s)
            for (int t = 0; t < T; ++t) {
                int hit = 0;
                for (int k = 0; k < K; ++k) {
                    int32_t e = topk[((size_t)s * T + t) * K + k];
                    if (e < 0 || e >= n_experts)
                        return -2;
                    if (e / per == d)
                        hit = 1;
                }
                if (!hit)
                    continue;
                if (fill >= cap)
                    return -1;
                const uint16_t *row = y + ((size_t)d * cap + fill) * H;
                float *a = acc + ((size_t)s * T + t) * H;
                if (!seen[(size_t)s * T + t]) {
                    for (size_t h = 0; h < H; ++h)
                        a[h] = orc_bf16_to_f32(row[h]);
                    seen[(size_t)s * T + t] = 1;
                } else {
                    for (size_t h = 0; h < H; ++h)
                        a[h] += orc_bf16_to_f32(row[h]);
                }
                ++fill;
            }
    }
    for (size_t i = 0; i < (size_t)n * T; ++i)
        for (size_t h = 0; h < H; ++h)
            out[i * H + h] = seen[i] ? orc_f32_to_bf16(acc[i * H + h]) : 0;
    return 0;
}

/* ---------- semaphore bookkeeping (the integer side of signal / wait) ---------- */

/* wait() is satisfied when the counter has reached the expected value; counters only
 * ever grow and wrap modulo 2^32, so "reached" is a signed distance test. */
int orc_sem_reached(uint32_t sem, uint32_t expected)
{
    return (int32_t)(sem - expected) >= 0;
}
