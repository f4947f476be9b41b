// Small kernels around the main ones: fills, state conversion, transposes, label check,
// negative class, clamp / argmax, copies.
// Part of the one translation unit tm_kernels.hip (included there, in this order).
#ifndef TM_KERNELS_UTIL_HPP_
#define TM_KERNELS_UTIL_HPP_

namespace tsetlin {

// ------------------------------------------------------------------------
// small utility kernels
// ------------------------------------------------------------------------

__global__ void k_fill_u32(uint32_t *p, int64_t nwords, uint32_t v)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride) p[i] = v;
}

// Initial TA states: state N or N+1 with probability 1/2, i.e. stored value
// 127 or 128.  One thread per (clause, literal word).
__global__ void k_init_state(Dims d, uint32_t *planes, uint32_t *inc)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)d.C * d.W) return;
    const int g = (int)(t / d.W);
    const int lw = (int)(t - (int64_t)g * d.W);
    const int fw = lw >= d.Wf ? lw - d.Wf : lw;
    const uint32_t valid = (fw == d.Wf - 1) ? d.tailmask : ~0u;
    const U4 r = draw(d.key, STREAM_INIT, 4u * (uint32_t)lw, (uint32_t)g, 0, 0);
    const uint32_t top = r.x & valid;
    uint32_t *p = planes + t * 8;
#pragma unroll
    for (int b = 0; b < 7; ++b) p[b] = ~top;
    p[7] = top;
    inc[t] = top;
}

// bytes (state - 1) -> bit planes; one thread per (clause, literal word)
__global__ void k_set_state(Dims d, const uint8_t *in, uint32_t *planes, uint32_t *inc)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)d.C * d.W) return;
    const int g = (int)(t / d.W);
    const int lw = (int)(t - (int64_t)g * d.W);
    const bool neg = lw >= d.Wf;
    const int fw = neg ? lw - d.Wf : lw;
    uint32_t p[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const uint8_t *row = in + (int64_t)g * 2 * d.o + (neg ? d.o : 0);
    for (int j = 0; j < 32; ++j) {
        const int f = fw * 32 + j;
        uint32_t stored = 127u; // padding automata: excluded, never touched
        if (f < d.o) {
            uint32_t v = row[f];
            if (v > (uint32_t)(2 * d.N - 1)) v = (uint32_t)(2 * d.N - 1);
            stored = v + (uint32_t)(128 - d.N);
        }
#pragma unroll
        for (int b = 0; b < 8; ++b) p[b] |= ((stored >> b) & 1u) << j;
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) planes[t * 8 + b] = p[b];
    inc[t] = p[7];
}

__global__ void k_get_state(Dims d, const uint32_t *planes, uint8_t *out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)d.C * d.W) return;
    const int g = (int)(t / d.W);
    const int lw = (int)(t - (int64_t)g * d.W);
    const bool neg = lw >= d.Wf;
    const int fw = neg ? lw - d.Wf : lw;
    uint32_t p[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) p[b] = planes[t * 8 + b];
    uint8_t *row = out + (int64_t)g * 2 * d.o + (neg ? d.o : 0);
    for (int j = 0; j < 32; ++j) {
        const int f = fw * 32 + j;
        if (f >= d.o) break;
        uint32_t stored = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) stored |= ((p[b] >> j) & 1u) << b;
        row[f] = (uint8_t)(stored - (uint32_t)(128 - d.N));
    }
}

// XT[fw][i] = X[i][fw], zero for q <= i < qp
__global__ void k_transpose_x(const uint32_t *X, uint32_t *XT, int64_t q, int64_t qp, int Wf)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= qp * Wf) return;
    const int fw = (int)(t / qp);
    const int64_t i = t - (int64_t)fw * qp;
    XT[t] = (i < q) ? X[i * Wf + fw] : 0u;
}

// labels must lie in [0, m) (regression mode: targets in [0, T], m = T + 1)
__global__ void k_check_labels(const int32_t *y, int64_t q, int m, int32_t *flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < q && (y[i] < 0 || y[i] >= m)) *flag = 1;
}

// sums[i][c] = clamp(sums[i][c], lo, T): lo = -T, or 0 in regression mode
__global__ void k_clamp(int32_t *sums, int64_t n, int lo, int T)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) sums[t] = min(max(sums[t], lo), T);
}

// pred[i] = lowest class index with the largest (already clamped) sum; in regression mode
// the clamped vote sum itself
__global__ void k_argmax(const int32_t *sums, int32_t *pred, int64_t q, int m, int regr)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= q) return;
    if (regr) {
        pred[i] = sums[i];
        return;
    }
    int best = 0;
    int32_t bv = sums[i * m];
    for (int c = 1; c < m; ++c) {
        const int32_t v = sums[i * m + c];
        if (v > bv) {
            bv = v;
            best = c;
        }
    }
    pred[i] = best;
}

// both of the above in one pass over the unclamped sums
__global__ void k_clamp_argmax(int32_t *sums, int32_t *pred, int64_t q, int m, int lo, int T, int regr)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= q) return;
    int best = 0;
    int32_t bv = 0;
    for (int c = 0; c < m; ++c) {
        const int32_t v = min(max(sums[i * m + c], lo), T);
        sums[i * m + c] = v;
        if (c == 0 || v > bv) {
            bv = v;
            best = c;
        }
    }
    pred[i] = regr ? bv : best;
}

// out[i][c] = tally[c][i]
__global__ void k_tally_out(const int32_t *tally, int32_t *out, int64_t q, int64_t qp, int m)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= q * m) return;
    const int64_t i = t / m;
    const int c = (int)(t - i * m);
    out[t] = tally[(int64_t)c * qp + i];
}

// dst[g][0..words) = src[g][0..words) for row strides that differ
__global__ void k_copy_rows(const uint32_t *src, int64_t src_stride, uint32_t *dst, int64_t dst_stride,
                            int64_t rows, int64_t words)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * words) return;
    const int64_t r = t / words, w = t - r * words;
    dst[r * dst_stride + w] = src[r * src_stride + w];
}

// fresh[g] = {plo, phi, slo, 0}: nothing outdated (0, 0, qp) or everything outdated (0, qp, qp)
__global__ void k_fresh_set(int32_t *fresh, int C, int qp, int all_stale)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < C) *reinterpret_cast<int4 *>(fresh + (int64_t)g * 4) = make_int4(0, all_stale ? qp : 0, qp, 0);
}

} // namespace tsetlin

#endif
