/*
 * SharpV two-stage pruning in float32 with every rounding written down ("canonical order").
 *
 * TEST INFRASTRUCTURE ONLY.  Plain scalar C, compiled with gcc -O2 -ffp-contract=off; it
 * shares no code with the GPU library and nothing in the product path may link or call it.
 *
 * Why it exists beside the float64 definition (sharpv_ref.py): the method turns floating
 * point scores into integer decisions (a per-frame kept count, a top-k set, a "cos < M"
 * mask).  For those decisions to be comparable bit for bit, both sides must take them in
 * the same precision and the same order of roundings.  The steps are the paper's, in the
 * paper's order (Sec. 3.1 Eq.1-6, Sec. 3.2 Eq.7); only the order of the float32 additions
 * inside each sum is pinned, as follows.
 *
 *   TREE32(p[0..31]):  for s = 16, 8, 4, 2, 1:  for l < s:  p[l] = p[l] + p[l+s];  result p[0].
 *
 *   ROWDOT(x, y, d)  (every inner product over the feature dimension):
 *       acc = +0
 *       for each block of 256 consecutive elements, ascending:
 *           for l in 0..31:  c[l] = +0;  for j in 0..7:  e = block*256 + 8*l + j
 *                                            if e < d:  c[l] = fmaf(x[e], y[e], c[l])
 *           acc = acc + TREE32(c)
 *
 *   COLMEAN(F[f][d])  (frame mean of Eq.2):  for each column c:
 *       p[g] = +0 (g < 32);  for i ascending:  p[i % 32] = p[i % 32] + F[i][c]
 *       mean[c] = TREE32(p) / (float) f            (kept in float32, never rounded to bf16)
 *
 *   SUM32(v[0..n-1])  (sums over the tokens of a frame / sequence):
 *       p[g] = +0;  for i ascending:  p[i % 32] = p[i % 32] + v[i];  result TREE32(p)
 *
 *   cos(xy, xx, yy) = den > 0 ? clamp(xy / den, -1, 1) : 0,  den = sqrtf(xx * yy)
 *   Dissim          = sqrtf(fmaxf(fmaf(-2, cos, 2), 0))                        (Eq.1, second form)
 *   I               = fmaf(w, S, T)                                            (Eq.4)
 *   r_t             = clamp(sqrtf(SUM32(T_i * T_i)) / (2 * sqrtf((float) f)), 0, 1)   (Eq.5/6)
 *   k_t             = clamp((int) floorf(r_t * (float) f + 0.5f), min_keep, f)
 *
 *   rotary re-encoding of a kept K row (Sec. 4.1, Implementation Details), pair (x, y), table entries c, s:
 *       x' = fmaf(x, c, y * s),  y' = fmaf(y, c, -(x * s)),  rounded once to the storage type
 *
 * bf16 inputs are widened exactly (bits << 16).  sqrtf and "/" are correctly rounded.
 * Identical rows give xx == yy == xy and sqrtf(xx*xx) == xx, hence cos == 1 and Dissim == 0
 * exactly (a repeated frame keeps nothing).  Inputs must be finite with xx*yy inside the
 * float32 range.
 *
 * Pins: tests/test_oracle_pins.py and tests/test_oracle_canon.py (agreement with the float64
 * definition inside the float32 error bound, closed forms, invariants, decision audit).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the outer loops (frames; tokens) run on. */
int sharpv_canon_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sets the number of threads of the outer loops (for timing the oracle on one core); n < 1 is ignored. */
void sharpv_canon_set_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

enum { CANON_F32 = 0, CANON_BF16 = 1 };

static float widen_at(const void* base, int dtype, size_t i) {
    if (dtype == CANON_F32) return ((const float*)base)[i];
    uint32_t u = (uint32_t)((const uint16_t*)base)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static void widen_row(const void* base, int dtype, size_t row, int d, float* out) {
    for (int e = 0; e < d; ++e) out[e] = widen_at(base, dtype, row * (size_t)d + (size_t)e);
}

static float tree32(float* p) {
    for (int s = 16; s >= 1; s >>= 1)
        for (int l = 0; l < s; ++l) p[l] = p[l] + p[l + s];
    return p[0];
}

float sharpv_canon_rowdot(const float* x, const float* y, int d) {
    float acc = 0.0f;
    for (int b0 = 0; b0 < d; b0 += 256) {
        float c[32];
        for (int l = 0; l < 32; ++l) {
            c[l] = 0.0f;
            for (int j = 0; j < 8; ++j) {
                int e = b0 + 8 * l + j;
                if (e < d) c[l] = fmaf(x[e], y[e], c[l]);
            }
        }
        acc = acc + tree32(c);
    }
    return acc;
}

float sharpv_canon_sum32(const float* v, int n) {
    float p[32];
    for (int g = 0; g < 32; ++g) p[g] = 0.0f;
    for (int i = 0; i < n; ++i) p[i % 32] = p[i % 32] + v[i];
    return tree32(p);
}

/* frame: [f][d] float32 (already widened) -> mean [d] */
void sharpv_canon_colmean(const float* frame, int f, int d, float* mean) {
    for (int c = 0; c < d; ++c) {
        float p[32];
        for (int g = 0; g < 32; ++g) p[g] = 0.0f;
        for (int i = 0; i < f; ++i) p[i % 32] = p[i % 32] + frame[(size_t)i * d + c];
        mean[c] = tree32(p) / (float)f;
    }
}

float sharpv_canon_cos(float xy, float xx, float yy) {
    float den = sqrtf(xx * yy);
    if (!(den > 0.0f)) return 0.0f;
    float c = xy / den;
    if (c > 1.0f) c = 1.0f;
    if (c < -1.0f) c = -1.0f;
    return c;
}

float sharpv_canon_dissim(float xy, float xx, float yy) {
    float q = fmaf(-2.0f, sharpv_canon_cos(xy, xx, yy), 2.0f);
    return sqrtf(fmaxf(q, 0.0f));
}

/* The rescaled cosine that Sec. 3.1 names as a possible stand-in for Eq.1 (with a fixed threshold K). */
float sharpv_canon_one_minus_cos(float xy, float xx, float yy) {
    return 1.0f - sharpv_canon_cos(xy, xx, yy);
}

static float measure_of(int measure, float xy, float xx, float yy) {
    return measure == 0 ? sharpv_canon_dissim(xy, xx, yy) : sharpv_canon_one_minus_cos(xy, xx, yy);
}

/*
 * Pre-LLM stage (Sec. 3.1).  feats [n_total][f][d]; frame_offsets [B+1].
 * Outputs: S, T, I [n_total*f]; ratio [n_total]; counts [n_total]; offsets [n_total+1];
 * idx (capacity n_total*f) global row indices ascending; out_feats (capacity of feats) kept rows.
 * mode 0: adaptive ratio + top-k (ties to the lowest index); mode 1: keep iff I >= K.
 * measure 0: S and T by Eq.1; measure 1: by one minus the cosine (mode 1 only).
 * Returns the total number of kept tokens, or -1 on a bad argument.
 */
long sharpv_canon_prune_tokens(const void* feats, int dtype, const int32_t* frame_offsets, int B,
                               int f, int d, float w, int mode, float K, int min_keep, int measure,
                               float* S, float* T, float* I, float* ratio,
                               int32_t* counts, int32_t* offsets, int32_t* idx, void* out_feats) {
    if (!feats || !frame_offsets || B < 1 || f < 1 || d < 1) return -1;
    if (measure < 0 || measure > 1 || (measure == 1 && mode != 1)) return -1;
    const int n_total = frame_offsets[B];
    const size_t esz = dtype == CANON_F32 ? 4 : 2;
    unsigned char* is_first = (unsigned char*)calloc((size_t)n_total + 1, 1);
    for (int b = 0; b < B; ++b)
        if (frame_offsets[b] < n_total) is_first[frame_offsets[b]] = 1;

#pragma omp parallel
    {
        float* cur = (float*)malloc((size_t)f * d * sizeof(float));
        float* prv = (float*)malloc((size_t)d * sizeof(float));
        float* mean = (float*)malloc((size_t)d * sizeof(float));
        float* tt = (float*)malloc((size_t)f * sizeof(float));
#pragma omp for schedule(dynamic, 1)
        for (int t = 0; t < n_total; ++t) {
            for (int i = 0; i < f; ++i) widen_row(feats, dtype, (size_t)t * f + i, d, cur + (size_t)i * d);
            sharpv_canon_colmean(cur, f, d, mean);                                   /* Eq.2: frame mean */
            const float mm = sharpv_canon_rowdot(mean, mean, d);
            for (int i = 0; i < f; ++i) {
                const float* x = cur + (size_t)i * d;
                const float xx = sharpv_canon_rowdot(x, x, d);
                const float xm = sharpv_canon_rowdot(x, mean, d);
                const float s = measure_of(measure, xm, xx, mm);                      /* Eq.2 */
                float tv;
                if (is_first[t]) {
                    tv = s;                                                          /* Eq.6: virtual preceding frame */
                } else {
                    widen_row(feats, dtype, (size_t)(t - 1) * f + i, d, prv);
                    const float pp = sharpv_canon_rowdot(prv, prv, d);
                    const float xp = sharpv_canon_rowdot(x, prv, d);
                    tv = measure_of(measure, xp, xx, pp);                             /* Eq.3 */
                }
                const size_t r = (size_t)t * f + i;
                S[r] = s;
                T[r] = tv;
                I[r] = fmaf(w, s, tv);                                               /* Eq.4 */
                tt[i] = tv * tv;
            }
            float rt = sqrtf(sharpv_canon_sum32(tt, f)) / (2.0f * sqrtf((float)f));  /* Eq.5 / Eq.6 */
            if (rt > 1.0f) rt = 1.0f;
            if (rt < 0.0f) rt = 0.0f;
            ratio[t] = rt;
            int k = 0;
            const float* It = I + (size_t)t * f;
            if (mode == 0) {
                float prod = rt * (float)f;
                k = (int)floorf(prod + 0.5f);
                if (k < min_keep) k = min_keep;
                if (k > f) k = f;
            } else {
                for (int i = 0; i < f; ++i) k += (It[i] >= K);
            }
            counts[t] = k;
        }
        free(cur); free(prv); free(mean); free(tt);
    }

    /* exclusive scan of the kept counts, then selection and compaction in stream order */
    offsets[0] = 0;
    for (int t = 0; t < n_total; ++t) offsets[t + 1] = offsets[t] + counts[t];
    for (int t = 0; t < n_total; ++t) {
        const float* It = I + (size_t)t * f;
        int32_t o = offsets[t];
        for (int i = 0; i < f; ++i) {
            int keep;
            if (mode == 0) {
                int rank = 0;   /* tokens ahead of i: higher score, or equal score and lower index */
                for (int j = 0; j < f; ++j) rank += (It[j] > It[i]) || (It[j] == It[i] && j < i);
                keep = rank < counts[t];
            } else {
                keep = It[i] >= K;
            }
            if (keep) {
                const size_t r = (size_t)t * f + i;
                idx[o] = (int32_t)r;
                memcpy((char*)out_feats + (size_t)o * d * esz, (const char*)feats + r * d * esz, (size_t)d * esz);
                ++o;
            }
        }
    }
    free(is_first);
    return offsets[n_total];
}

/*
 * Intra-LLM stage for one layer (Sec. 3.2, Eq.7).  hidden [S][d]; orig [n_vis][d]; Kc, Vc [H][S][D]
 * contiguous.  Visual token p of sequence b is at packed position seq_offsets[b] + vis_start[b] +
 * (p - vis_offsets[b]).  kv_mode 0: token discarded iff cos < M.  kv_mode 1: all visual tokens of a
 * sequence discarded iff mean_cos[b] = SUM32(cos over the sequence's visual tokens) / n_b < M.
 * Outputs: cosv [n_vis]; mean_cos [B]; out_idx (capacity S) kept packed positions ascending;
 * out_count [B]; K_out, V_out [H][S_kept][D] contiguous.  Returns S_kept or -1.
 */
long sharpv_canon_prune_kv(const void* hidden, const void* orig, const void* Kc, const void* Vc, int dtype,
                           const int32_t* seq_offsets, const int32_t* vis_start, const int32_t* vis_offsets,
                           int B, int d, int H, int D, float M, int kv_mode,
                           float* cosv, float* mean_cos, int32_t* out_idx, int32_t* out_count,
                           void* K_out, void* V_out) {
    if (!hidden || !orig || !seq_offsets || !vis_start || !vis_offsets || B < 1) return -1;
    const int S = seq_offsets[B];
    const size_t esz = dtype == CANON_F32 ? 4 : 2;
    unsigned char* keep = (unsigned char*)malloc((size_t)S + 1);
    memset(keep, 1, (size_t)S + 1);                     /* system / instruction tokens are always kept */
    for (int b = 0; b < B; ++b) {
        const int lo = vis_offsets[b], hi = vis_offsets[b + 1];
        const int p0 = seq_offsets[b] + vis_start[b];
#pragma omp parallel
        {
            float* h = (float*)malloc((size_t)d * sizeof(float));
            float* o = (float*)malloc((size_t)d * sizeof(float));
#pragma omp for schedule(static)
            for (int p = lo; p < hi; ++p) {
                widen_row(hidden, dtype, (size_t)(p0 + (p - lo)), d, h);
                widen_row(orig, dtype, (size_t)p, d, o);
                const float hh = sharpv_canon_rowdot(h, h, d);
                const float oo = sharpv_canon_rowdot(o, o, d);
                const float ho = sharpv_canon_rowdot(h, o, d);
                cosv[p] = sharpv_canon_cos(ho, hh, oo);
            }
            free(h); free(o);
        }
        mean_cos[b] = hi > lo ? sharpv_canon_sum32(cosv + lo, hi - lo) / (float)(hi - lo) : 0.0f;
        for (int p = lo; p < hi; ++p) {
            int discard = kv_mode == 0 ? (cosv[p] < M) : (mean_cos[b] < M);          /* Eq.7 */
            if (discard) keep[p0 + (p - lo)] = 0;
        }
    }
    long n_kept = 0;
    for (int b = 0; b < B; ++b) {
        int c = 0;
        for (int s = seq_offsets[b]; s < seq_offsets[b + 1]; ++s)
            if (keep[s]) { out_idx[n_kept + c] = s; ++c; }
        out_count[b] = c;
        n_kept += c;
    }
    if (Kc && Vc && K_out && V_out) {
        for (int hh = 0; hh < H; ++hh)
            for (long j = 0; j < n_kept; ++j) {
                const size_t src = ((size_t)hh * S + (size_t)out_idx[j]) * D * esz;
                const size_t dst = ((size_t)hh * n_kept + (size_t)j) * D * esz;
                memcpy((char*)K_out + dst, (const char*)Kc + src, (size_t)D * esz);
                memcpy((char*)V_out + dst, (const char*)Vc + src, (size_t)D * esz);
            }
    }
    free(keep);
    return n_kept;
}

/* ------------------------------------------------------------------------------------------------
 * Eq.7 on a sequence that earlier layers have already thinned out (Sec. 3.2, Degradation-Aware Pruning).
 *
 * hidden [S][d], K / V [H][S][D] hold the positions still alive; orig_row[s] is the row of orig
 * [n_orig][d] behind position s, or -1 (anything outside [0, n_orig) counts as -1) for a system /
 * instruction position, which is always kept.  A visual position is discarded iff its cosine < M.
 * Outputs: cosv [S] (written at visual positions only); out_idx kept positions ascending; out_count [B];
 * out_orig_row = orig_row of the kept positions; K_out, V_out [H][S_kept][D].  Returns S_kept or -1.
 */
long sharpv_canon_prune_kv_mapped(const void* hidden, const void* orig, const int32_t* orig_row, const void* Kc,
                                  const void* Vc, int dtype, const int32_t* seq_offsets, int B, int n_orig, int d,
                                  int H, int D, float M, float* cosv, int32_t* out_idx, int32_t* out_count,
                                  int32_t* out_orig_row, void* K_out, void* V_out) {
    if (!hidden || !orig || !orig_row || !seq_offsets || B < 1) return -1;
    const int S = seq_offsets[B];
    const size_t esz = dtype == CANON_F32 ? 4 : 2;
    unsigned char* keep = (unsigned char*)malloc((size_t)S + 1);
    memset(keep, 1, (size_t)S + 1);
#pragma omp parallel
    {
        float* h = (float*)malloc((size_t)d * sizeof(float));
        float* o = (float*)malloc((size_t)d * sizeof(float));
#pragma omp for schedule(static)
        for (int s = 0; s < S; ++s) {
            const int p = orig_row[s];
            if (p < 0 || p >= n_orig) continue;
            widen_row(hidden, dtype, (size_t)s, d, h);
            widen_row(orig, dtype, (size_t)p, d, o);
            const float hh = sharpv_canon_rowdot(h, h, d);
            const float oo = sharpv_canon_rowdot(o, o, d);
            const float ho = sharpv_canon_rowdot(h, o, d);
            const float c = sharpv_canon_cos(ho, hh, oo);
            if (cosv) cosv[s] = c;
            if (c < M) keep[s] = 0;                                                   /* Eq.7 */
        }
        free(h); free(o);
    }
    long n_kept = 0;
    for (int b = 0; b < B; ++b) {
        int c = 0;
        for (int s = seq_offsets[b]; s < seq_offsets[b + 1]; ++s)
            if (keep[s]) {
                const int p = orig_row[s];
                out_idx[n_kept + c] = s;
                if (out_orig_row) out_orig_row[n_kept + c] = (p < 0 || p >= n_orig) ? -1 : p;
                ++c;
            }
        out_count[b] = c;
        n_kept += c;
    }
    if (Kc && Vc && K_out && V_out) {
        for (int hh = 0; hh < H; ++hh)
            for (long j = 0; j < n_kept; ++j) {
                const size_t src = ((size_t)hh * S + (size_t)out_idx[j]) * D * esz;
                const size_t dst = ((size_t)hh * n_kept + (size_t)j) * D * esz;
                memcpy((char*)K_out + dst, (const char*)Kc + src, (size_t)D * esz);
                memcpy((char*)V_out + dst, (const char*)Vc + src, (size_t)D * esz);
            }
    }
    free(keep);
    return n_kept;
}

/* ------------------------------------------------------------------------------------------------
 * Rotary re-encoding of the compacted K cache (Sec. 4.1, Implementation Details), in place.
 *
 * K_rows [H][n_kept][D] are the kept K rows in stream order, out_idx their packed positions.  The
 * j-th kept row of a sequence that sat at position p of that sequence is turned back by
 * delta = p - j steps:  with c = cos_tab[delta][i], s = sin_tab[delta][i] (tables [rope_len][D/2] from the
 * caller) and (x, y) the i-th pair of the row (layout 0: elements i and i + D/2; layout 1: 2i and 2i+1)
 *     x' = fmaf(x, c, y * s)        y' = fmaf(y, c, -(x * s))
 * in float32 (the two products y*s and x*s rounded on their own), then rounded to the storage type
 * (bf16: to nearest, ties to even).  Returns 0, or -1 for a bad argument or a delta >= rope_len.
 */
static uint16_t f32_to_bf16_rne(float v) {
    uint32_t u;
    memcpy(&u, &v, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int sharpv_canon_rope_reencode(void* K_rows, int dtype, const int32_t* out_idx, long n_kept,
                               const int32_t* seq_offsets, int B, int H, int D,
                               const float* cos_tab, const float* sin_tab, int rope_len, int layout) {
    if (!K_rows || !out_idx || !seq_offsets || !cos_tab || !sin_tab || B < 1 || D < 2 || (D & 1)) return -1;
    if (layout != 0 && layout != 1) return -1;
    const int half = D / 2;
    int seq = 0, rank = 0;
    for (long j = 0; j < n_kept; ++j) {
        const int s = out_idx[j];
        while (seq + 1 < B && s >= seq_offsets[seq + 1]) { ++seq; rank = 0; }
        const int delta = (s - seq_offsets[seq]) - rank;
        if (delta < 0 || delta >= rope_len) return -1;
        const float* ct = cos_tab + (size_t)delta * half;
        const float* st = sin_tab + (size_t)delta * half;
        for (int h = 0; h < H; ++h) {
            const size_t row = ((size_t)h * (size_t)n_kept + (size_t)j) * (size_t)D;
            for (int i = 0; i < half; ++i) {
                const size_t ia = row + (size_t)(layout == 0 ? i : 2 * i);
                const size_t ib = row + (size_t)(layout == 0 ? i + half : 2 * i + 1);
                float x, y;
                if (dtype == CANON_F32) { x = ((float*)K_rows)[ia]; y = ((float*)K_rows)[ib]; }
                else {
                    uint32_t ux = (uint32_t)((uint16_t*)K_rows)[ia] << 16, uy = (uint32_t)((uint16_t*)K_rows)[ib] << 16;
                    memcpy(&x, &ux, 4); memcpy(&y, &uy, 4);
                }
                const float ys = y * st[i];
                const float xs = x * st[i];
                const float xn = fmaf(x, ct[i], ys);
                const float yn = fmaf(y, ct[i], -xs);
                if (dtype == CANON_F32) { ((float*)K_rows)[ia] = xn; ((float*)K_rows)[ib] = yn; }
                else { ((uint16_t*)K_rows)[ia] = f32_to_bf16_rne(xn); ((uint16_t*)K_rows)[ib] = f32_to_bf16_rne(yn); }
            }
        }
        ++rank;
    }
    return 0;
}
