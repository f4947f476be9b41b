// HIP kernels and C boundary of the asynchronous Tsetlin machine (gfx950).
//
// Memory layout (all device memory is caller-owned):
//   state buffer   planes uint32 [C][W][8]  bit-sliced TA counters, W = 2*Wf literal words
//                  inc    uint32 [C][W]     include masks (= plane 7), compact copy for evaluation
//   train workspace
//                  tally  int32  [m][qp]    voting tallies, qp = q rounded up to 64
//                  ostar  uint32 [C][Qw]    previous clause outputs, 1 bit per (clause, example), Qw = qp/32
//                  XT     uint32 [Wf][qp]   transposed features (word-major) for lane = example evaluation
//                  XB     uint32 [2o+1][QW] literals as bit rows over the examples (row 2o all ones), QW = 64*ceil(q/2048)
//                  lits   uint32 [C][128]   literal lists of the clauses, nlit int32 [C] their lengths
//                  negcls int32  [qp]       class trained towards 0 for each example, this epoch
//                  gate   int32  [m][qp]    per class and launch: ascending list of (example << 1 | target) whose gate can open
//                  fresh  int32  [C][4]     per clause: example ranges whose stored outputs may be outdated
//                  order  int32  [C]        launch order of the clauses (outdated ones first)
//                  counters uint64 [64][8] interleaved event counters, flag int32
//   literal word lw < Wf holds x_(32 lw + j), literal word Wf + fw holds NOT x_(32 fw + j).
//
// Three evaluation layouts are used:
//   k_eval_sparse lane = 32 examples : one clause per wavefront at a time, one word of XB
//            per included literal; votes counted bit-sliced (tally pre-calculation and
//            inference with a workspace).
//   k_eval_* lane = clause : include masks in VGPRs, example words arrive through
//            scalar loads, one bit-select per feature word and pair; clause votes are
//            summed with wave ballot + popcount (inference, tally pre-calculation).
//   k_train  one wavefront = one clause (Algorithm 1 gives every clause its own
//            thread); lane = gate-list entry for the gates, lane = literal word for
//            feedback, lane = example for the evaluation of a block of 64 examples.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <math.h>
#include <new>
#include <stdint.h>
#include <string.h>
#include <vector>

#include "../../include/tm.h"
#include "tm_device.hpp"

namespace tsetlin {

struct Dims {
    int m, n, o, N, T, C, Wf, W;
    uint32_t thr;      // 16-bit threshold: P(u < thr) = 1/s
    uint32_t boost;    // ~0 if true positives are boosted (strong Type I event certain), else 0
    uint32_t tailmask; // valid bits of the last feature word
    RngKey key;
};

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

__global__ void k_check_labels(const int32_t *y, int64_t q, int m, int32_t *flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < q && (y[i] < 0 || y[i] >= m)) *flag = 1;
}

// The class trained towards output 0 for example i in this epoch: uniform over
// the m-1 classes other than y_i, a function of (seed, epoch, i) only so that
// all clauses agree without communicating.
__global__ void k_negcls(Dims d, const int32_t *y, int32_t *negcls, int64_t q, int64_t qp, uint32_t epoch)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= qp) return;
    int32_t r = -1;
    if (i < q) {
        const U4 u = draw(d.key, STREAM_NEGCLASS, 0, 0, (uint64_t)i, epoch);
        const int32_t dd = (int32_t)(((uint64_t)u.x * (uint64_t)(d.m - 1)) >> 32);
        r = dd + (dd >= y[i] ? 1 : 0);
    }
    negcls[i] = r;
}

// sums[i][c] = clamp(sums[i][c], -T, T)
__global__ void k_clamp(int32_t *sums, int64_t n, int T)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) sums[t] = min(max(sums[t], -T), T);
}

// pred[i] = lowest class index with the largest (already clamped) sum
__global__ void k_argmax(const int32_t *sums, int32_t *pred, int64_t q, int m)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= q) return;
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
__global__ void k_clamp_argmax(int32_t *sums, int32_t *pred, int64_t q, int m, int T)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= q) return;
    int best = 0;
    int32_t bv = 0;
    for (int c = 0; c < m; ++c) {
        const int32_t v = min(max(sums[i * m + c], -T), T);
        sums[i * m + c] = v;
        if (c == 0 || v > bv) {
            bv = v;
            best = c;
        }
    }
    pred[i] = best;
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

// What a launch of the training kernel over the examples [i_begin, i_end) needs: two stable
// compactions.
//
// Task c < m: gate list of class c = the examples of the range, ascending, whose gate can
// open for a clause of c, packed as (example << 1 | target): target 1 where y_i = c,
// target 0 where c is the class drawn against y_i, and error e > 0 under the tally as it
// stands now (or under the snapshot vhat).  The examples with e = 0 are left out: their
// gate probability e/2T is 0, so a clause that read this tally would not act, and reading
// a tally that is one launch old is within the method's premise of outdated tallies
// (Section 3.1).  The clause re-reads the tally of a listed example when it gets there.
// ngate[c] receives the length; counter 4 the number of (clause, example) pairs of the
// range whose class is trained for the example.
//
// Task m: launch order of the clauses.  Those that start the launch with outdated stored
// outputs sweep every block of the range and go first (ascending), so that they do not end
// up alone at the tail of the launch; the others fill the order from its end.
//
// The items of a task (examples of the range, clauses) are cut into segments of
// PREP_SEG, one workgroup of 1024 each, so that the loads of the whole range are in flight
// at once; the kernel runs twice: the first run leaves the number of flagged items of
// every segment in seg_cnt, the second run places them.
struct PrepArgs {
    const int32_t *y, *negcls, *tally, *vhat, *fresh;
    int32_t *gate, *ngate, *order, *seg_cnt; // seg_cnt [m + 1][segs][2]
    unsigned long long *counters;
    int i_begin, i_end, qp, m, n, C, T, segs;
};

constexpr int COUNTER_SETS = 64; // interleaved copies of the 8 event counters
constexpr int PREP_ROUNDS = 4;   // rounds of 1024 items per segment
constexpr int PREP_SEG = 1024 * PREP_ROUNDS;

template <bool PLACE>
__global__ __launch_bounds__(1024) void k_launch_prep(const PrepArgs a)
{
    __shared__ int cnt[PREP_ROUNDS * 16][2]; // [round][wavefront] x [front, back]
    __shared__ int seg_base[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int task = blockIdx.y, seg = blockIdx.x;
    const bool ordering = task == a.m;
    const int c = task;
    const int lo = ordering ? 0 : a.i_begin, hi = ordering ? a.C : a.i_end;
    const int p0 = lo + seg * PREP_SEG;
    if (p0 >= hi) return; // the grid is sized for the longer of the two kinds of task
    const int32_t *vsrc = a.vhat ? a.vhat + c : a.tally + (int64_t)c * a.qp;
    const int64_t vstride = a.vhat ? a.m : 1;
    int32_t *sc = a.seg_cnt + ((int64_t)task * a.segs) * 2;
    // an item past the end is read as the last item (no branch around the loads) and dropped
    bool f[PREP_ROUNDS], bk[PREP_ROUNDS], tg[PREP_ROUNDS];
    int n_seen = 0;
#pragma unroll
    for (int r = 0; r < PREP_ROUNDS; ++r) {
        const int t = p0 + r * 1024 + tid;
        const bool live = t < hi;
        const int tc = min(t, hi - 1);
        bk[r] = tg[r] = false;
        if (ordering) {
            const int4 fr = *reinterpret_cast<const int4 *>(a.fresh + (int64_t)tc * 4);
            const bool stale = (fr.x < fr.y && fr.x < a.i_end && fr.y > a.i_begin) || (fr.z < a.i_end);
            f[r] = live && stale;
            bk[r] = live && !stale;
        } else {
            const int yy = a.y[tc], ng = a.negcls[tc], v = vsrc[(int64_t)tc * vstride];
            tg[r] = live && yy == c;
            const bool match = live && (tg[r] || ng == c);
            const int vc = min(max(v, -a.T), a.T);
            n_seen += match ? 1 : 0;
            f[r] = match && (tg[r] ? a.T - vc : a.T + vc) > 0; // Algorithm 1: error of the recorded vote sum
        }
    }
    uint64_t bf[PREP_ROUNDS], bb[PREP_ROUNDS];
#pragma unroll
    for (int r = 0; r < PREP_ROUNDS; ++r) {
        bf[r] = ballot(f[r]);
        bb[r] = ballot(bk[r]);
        if (lane == 0) {
            cnt[r * 16 + wave][0] = __builtin_popcountll(bf[r]);
            cnt[r * 16 + wave][1] = __builtin_popcountll(bb[r]);
        }
    }
    if (PLACE && tid < 2) { // where this segment starts: the flagged items of the segments before it
        int sum = 0;
        for (int k = 0; k < seg; ++k) sum += sc[k * 2 + tid];
        seg_base[tid] = sum;
    }
    __syncthreads();
    // flagged items of the (round, wavefront) slots before the own one, and of the whole segment
    int before_f = 0, before_b = 0, all_f = 0, all_b = 0;
    if (wave == 0) {
        const int vf = cnt[lane][0], vb = cnt[lane][1]; // PREP_ROUNDS * 16 = 64 slots: one per lane
        int inf = vf, inb = vb;
#pragma unroll
        for (int dlt = 1; dlt < 64; dlt <<= 1) {
            const int tf = __shfl_up(inf, dlt, 64), tb = __shfl_up(inb, dlt, 64);
            if (lane >= dlt) {
                inf += tf;
                inb += tb;
            }
        }
        all_f = __shfl(inf, 63, 64);
        all_b = __shfl(inb, 63, 64);
        if (!PLACE) {
            if (lane == 0) {
                sc[seg * 2] = all_f;
                sc[seg * 2 + 1] = all_b;
            }
        } else {
            cnt[lane][0] = inf - vf;
            cnt[lane][1] = inb - vb;
        }
    }
    if (!PLACE) {
        if (!ordering) { // pairs of the range whose class is trained for the example
            for (int sh = 32; sh > 0; sh >>= 1) n_seen += __shfl_down(n_seen, sh, 64);
            if (lane == 0 && n_seen)
                atomicAdd(&a.counters[((seg * 16 + wave) & (COUNTER_SETS - 1)) * 8 + 4],
                          (unsigned long long)n_seen * (unsigned long long)a.n);
        }
        return;
    }
    __syncthreads();
    int32_t *out = ordering ? a.order : a.gate + (int64_t)c * a.qp;
#pragma unroll
    for (int r = 0; r < PREP_ROUNDS; ++r) {
        const int t = p0 + r * 1024 + tid;
        const int value = ordering ? t : ((t << 1) | (tg[r] ? 1 : 0));
        before_f = seg_base[0] + cnt[r * 16 + wave][0];
        before_b = seg_base[1] + cnt[r * 16 + wave][1];
        if (f[r])
            out[before_f + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bf[r] >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)bf[r], 0u))] = value;
        if (bk[r])
            out[a.C - 1 - (before_b + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bb[r] >> 32),
                                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)bb[r], 0u)))] = value;
    }
    // the last segment of a gate list knows its length
    if (!ordering && wave == 0 && lane == 0 && p0 + PREP_SEG >= hi) a.ngate[c] = seg_base[0] + all_f;
}

// ------------------------------------------------------------------------
// k_eval: clause evaluation, lane = clause   (Eq. 1, Eq. 3, Section 3.1)
// ------------------------------------------------------------------------

// inc  [C][W] include masks, X [q][Wf] examples (both read-only, passed as
// restrict kernel arguments so that the example words can be fetched with
// scalar loads); bits [C][bits_stride] clause outputs or null; signed vote
// sums are atomically added to acc[i*acc_si + c*acc_sc] unless acc is null.
struct EvalArgs {
    int64_t q;
    int Wf, W, C, n, m;
    int64_t bits_stride;
    int64_t acc_si, acc_sc;
    int64_t ex_per_wave; // multiple of 256
};

// A wavefront owns 64 consecutive clauses (a "tile") and a range of examples.
// The words of one example are wave-uniform and come in through scalar loads,
// so the violation test of a feature word for 64 clauses,
//   (inc_neg & x) | (inc_pos & ~x),
// is a single bit-select with the scalar x as selector.  Votes are summed with
// ballot + popcount against the polarity masks (odd clause index = positive).

// Vote of the clauses of class `cc` in this tile for one example.
__device__ __forceinline__ int tile_vote(uint64_t satisfied, uint64_t cmpos, uint64_t cmneg)
{
    return __builtin_popcountll(satisfied & cmpos) - __builtin_popcountll(satisfied & cmneg);
}

// Violation words of `ne` consecutive examples starting at row `base` for the 64 clauses
// of a wavefront whose masks sit in mn/mp (resident variant): post(e, viol) is called for
// e = 0..ne-1 in order.  The first nf examples may be read CH words wide (a row shorter
// than CH is over-read into the next row, where the surplus masks are 0); they go through
// two row buffers in turn, the row of the next example being requested before the current
// one is consumed, so that the scalar-load latency hides behind the bit operations.  The
// remaining examples (the last row of X when it is shorter than CH words) are read guarded.
template <int CH, typename Post>
__device__ __forceinline__ void resident_rows(const uint32_t *__restrict__ X, int Wf, int64_t base, int ne, int nf,
                                              const uint32_t (&mn)[CH], const uint32_t (&mp)[CH], Post &&post)
{
    if (nf > 0) {
        auto load = [&](uint32_t (&x)[CH], int e) {
            const int64_t ir = base + min(e, nf - 1); // clamped: a surplus request re-reads a valid row
            const uint32_t *xr = X + ir * Wf;         // wave-uniform
#pragma unroll
            for (int w = 0; w < CH; ++w) x[w] = xr[w];
        };
        auto consume = [&](const uint32_t (&x)[CH], int e) {
            uint32_t viol = 0;
#pragma unroll
            for (int w = 0; w < CH; ++w) viol |= bitselect(x[w], mn[w], mp[w]); // negated literal violated where x = 1, plain where x = 0
            post(e, viol);
        };
        uint32_t xa[CH], xb[CH];
        load(xa, 0);
        int e = 0;
        for (; e + 1 < nf; e += 2) {
            load(xb, e + 1);
            consume(xa, e);
            load(xa, e + 2);
            consume(xb, e + 1);
        }
        if (e < nf) consume(xa, e);
    }
    for (int e = max(nf, 0); e < ne; ++e) {
        const uint32_t *xr = X + (base + e) * Wf;
        uint32_t viol = 0;
#pragma unroll
        for (int w = 0; w < CH; ++w) {
            if (w < Wf) viol |= bitselect(xr[w], mn[w], mp[w]);
        }
        post(e, viol);
    }
}

// Resident variant, Wf <= CH <= 32: both mask halves of the tile stay in 2*CH
// VGPRs for the whole range of examples.  Rows of X are read CH words wide; a
// row shorter than CH is over-read into the next row (the surplus masks are 0),
// except for the last row of X, which takes a guarded path.
template <int CH, bool BITS, bool ACC>
__global__ __launch_bounds__(64) void k_eval_resident(const uint32_t *__restrict__ inc,
                                                      const uint32_t *__restrict__ X, uint32_t *__restrict__ bits,
                                                      int32_t *__restrict__ acc, const EvalArgs a)
{
    const int lane = threadIdx.x;
    const int tile = blockIdx.x;
    const int g = tile * 64 + lane;
    const bool gv = g < a.C;
    const int64_t e_begin = (int64_t)blockIdx.y * a.ex_per_wave;
    const int64_t e_end = min(a.q, e_begin + a.ex_per_wave);
    if (e_begin >= e_end) return;

    const uint32_t *mrow = inc + (int64_t)(gv ? g : 0) * a.W;
    uint32_t mp[CH], mn[CH];
#pragma unroll
    for (int w = 0; w < CH; ++w) {
        const bool ok = gv && (w < a.Wf);
        const int wi = w < a.Wf ? w : 0;
        const uint32_t vp = mrow[wi], vn = mrow[a.Wf + wi];
        mp[w] = ok ? vp : 0u;
        mn[w] = ok ? vn : 0u;
    }

    const int c_first = (tile * 64) / a.n;
    const int c_last = (min(a.C, tile * 64 + 64) - 1) / a.n;
    const bool one_class = (c_first == c_last);
    const int my_class = gv ? g / a.n : -1;
    const uint64_t cm0 = ballot(my_class == c_first);
    const uint64_t cmpos0 = cm0 & 0xAAAAAAAAAAAAAAAAull, cmneg0 = cm0 & 0x5555555555555555ull;
    const int64_t safe_end = (a.Wf == CH) ? e_end : min(e_end, a.q - 1);

    for (int64_t b0 = e_begin; b0 < e_end; b0 += 64) {
        const int nb = (int)min((int64_t)64, e_end - b0);
        uint32_t sat[2] = {0u, 0u}; // bit e: this lane's clause is satisfied by example b0 + 32*h + e
        int accv = 0;               // lane e: vote of class c_first in this tile for example b0 + e
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t base = b0 + 32 * h;
            const int ne = min(32, nb - 32 * h);
            const int nf = (int)min((int64_t)ne, safe_end - base); // examples whose rows may be read CH words wide
            auto post = [&](int e, uint32_t viol) {
                const bool ok = (viol == 0u);
                if (BITS || !one_class) sat[h] |= ok ? (1u << e) : 0u;
                if (ACC) {
                    const int s = tile_vote(ballot(ok), cmpos0, cmneg0);
                    accv = (lane == 32 * h + e) ? s : accv;
                }
            };
            resident_rows<CH>(X, a.Wf, base, ne, nf, mn, mp, post);
        }
        if (BITS && gv) {
            bits[(int64_t)g * a.bits_stride + (b0 >> 5)] = sat[0];
            if (nb > 32) bits[(int64_t)g * a.bits_stride + (b0 >> 5) + 1] = sat[1];
        }
        if (ACC) {
            const int64_t i = b0 + lane;
            if (lane < nb && accv != 0) atomicAdd(acc + i * a.acc_si + (int64_t)c_first * a.acc_sc, accv);
            if (!one_class) { // tiles that straddle class boundaries: remaining classes from the stored bits
                for (int cc = c_first + 1; cc <= c_last; ++cc) {
                    const uint64_t cm = ballot(my_class == cc);
                    const uint64_t cmpos = cm & 0xAAAAAAAAAAAAAAAAull, cmneg = cm & 0x5555555555555555ull;
                    int av = 0;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int ne = min(32, nb - 32 * h);
                        for (int e = 0; e < ne; ++e) {
                            const int s = tile_vote(ballot(((sat[h] >> e) & 1u) != 0u), cmpos, cmneg);
                            av = (lane == 32 * h + e) ? s : av;
                        }
                    }
                    if (lane < nb && av != 0) atomicAdd(acc + i * a.acc_si + (int64_t)cc * a.acc_sc, av);
                }
            }
        }
    }
}

// Streaming variant for masks wider than the register budget (Wf > 32): the
// masks are streamed in chunks of 32 feature words per batch of 256 examples;
// a lane keeps one "violated" flag bit per example of the batch.
__global__ __launch_bounds__(64) void k_eval_stream(const uint32_t *__restrict__ inc, const uint32_t *__restrict__ X,
                                                    uint32_t *__restrict__ bits, int32_t *__restrict__ acc,
                                                    const EvalArgs a)
{
    constexpr int CH = 32;
    const int lane = threadIdx.x;
    const int tile = blockIdx.x;
    const int g = tile * 64 + lane;
    const bool gv = g < a.C;
    const int64_t e_begin = (int64_t)blockIdx.y * a.ex_per_wave;
    const int64_t e_end = min(a.q, e_begin + a.ex_per_wave);
    if (e_begin >= e_end) return;

    const int nch = (a.Wf + CH - 1) / CH;
    const uint32_t *mrow = inc + (int64_t)(gv ? g : 0) * a.W;
    const int c_first = (tile * 64) / a.n;
    const int c_last = (min(a.C, tile * 64 + 64) - 1) / a.n;
    const int my_class = gv ? g / a.n : -1;

    for (int64_t b0 = e_begin; b0 < e_end; b0 += 256) {
        const int nb = (int)min((int64_t)256, e_end - b0);
        uint32_t flags[8];
#pragma unroll
        for (int fb = 0; fb < 8; ++fb) flags[fb] = 0;

        for (int ch = 0; ch < nch; ++ch) {
            const int w0 = ch * CH;
            uint32_t mp[CH], mn[CH];
#pragma unroll
            for (int w = 0; w < CH; ++w) {
                const bool ok = gv && (w0 + w < a.Wf);
                const int wi = (w0 + w < a.Wf) ? w0 + w : 0;
                const uint32_t vp = mrow[wi], vn = mrow[a.Wf + wi];
                mp[w] = ok ? vp : 0u;
                mn[w] = ok ? vn : 0u;
            }
            const bool full = (w0 + CH <= a.Wf);
#pragma unroll
            for (int fb = 0; fb < 8; ++fb) {
                const int ne = min(32, nb - fb * 32);
                if (ne <= 0) continue;
                if (full) {
                    // two row buffers in turn: the next example's words are requested before the
                    // current ones are consumed (scalar-load latency hides behind the bit operations)
                    auto load = [&](uint32_t (&x)[CH], int e) {
                        const int ee = min(e, ne - 1); // a surplus request re-reads the last row
                        const uint32_t *xr = X + (b0 + fb * 32 + ee) * a.Wf + w0; // wave-uniform
#pragma unroll
                        for (int w = 0; w < CH; ++w) x[w] = xr[w];
                    };
                    auto consume = [&](const uint32_t (&x)[CH], int e) {
                        uint32_t viol = 0;
#pragma unroll
                        for (int w = 0; w < CH; ++w) viol |= bitselect(x[w], mn[w], mp[w]); // negated literal violated where x = 1, plain where x = 0
                        flags[fb] |= (viol != 0u) ? (1u << e) : 0u;
                    };
                    uint32_t xa[CH], xb[CH];
                    load(xa, 0);
                    int e = 0;
                    for (; e + 1 < ne; e += 2) {
                        load(xb, e + 1);
                        consume(xa, e);
                        load(xa, e + 2);
                        consume(xb, e + 1);
                    }
                    if (e < ne) consume(xa, e);
                } else {
                    for (int e = 0; e < ne; ++e) {
                        const uint32_t *xr = X + (b0 + fb * 32 + e) * a.Wf + w0; // wave-uniform
                        uint32_t viol = 0;
#pragma unroll
                        for (int w = 0; w < CH; ++w) {
                            if (w0 + w < a.Wf) viol |= bitselect(xr[w], mn[w], mp[w]);
                        }
                        flags[fb] |= (viol != 0u) ? (1u << e) : 0u;
                    }
                }
            }
        }

        if (bits) {
#pragma unroll
            for (int fb = 0; fb < 8; ++fb) {
                const int ne = min(32, nb - fb * 32);
                if (ne > 0 && gv) {
                    const uint32_t lowmask = ne >= 32 ? ~0u : ((1u << ne) - 1u);
                    bits[(int64_t)g * a.bits_stride + (b0 >> 5) + fb] = ~flags[fb] & lowmask;
                }
            }
        }

        if (acc) {
            for (int cc = c_first; cc <= c_last; ++cc) {
                const uint64_t cm = ballot(my_class == cc);
                const uint64_t cmpos = cm & 0xAAAAAAAAAAAAAAAAull; // odd index within class: positive polarity
                const uint64_t cmneg = cm & 0x5555555555555555ull;
                int accv[4] = {0, 0, 0, 0};
#pragma unroll
                for (int fb = 0; fb < 8; ++fb) {
                    const int ne = min(32, nb - fb * 32);
                    for (int e = 0; e < ne; ++e) {
                        const int s = tile_vote(ballot(((flags[fb] >> e) & 1u) == 0u), cmpos, cmneg);
                        accv[fb >> 1] = (lane == (fb & 1) * 32 + e) ? s : accv[fb >> 1];
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int64_t i = b0 + k * 64 + lane;
                    if (i < e_end && accv[k] != 0) atomicAdd(acc + i * a.acc_si + (int64_t)cc * a.acc_sc, accv[k]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------
// k_eval_sparse: clause evaluation from literal lists, lane = 32 examples
// ------------------------------------------------------------------------
//
// A trained clause includes a few dozen of its 2o literals, so its output on 32 examples
// is the AND of that many 32-bit words when the literals are stored literal-major:
// XB [2o + 1][QW] uint32, bit b of word w of row k = literal k of example 32 w + b (rows
// 0..o-1 the features, rows o..2o-1 their negations); row 2o is all ones (padding of
// literal lists), QW = words per row, a multiple of 64.  A wavefront
// then evaluates one clause on 2048 examples with one coalesced 256-byte load and one
// bit operation per included literal - against one operation per feature WORD and
// example in the lane = clause kernels above.  This is the GPU counterpart of indexing
// clauses by their literals.  An untrained clause includes about half of all literals,
// but then some literal is false on every example after a few loads and the loop stops.

constexpr int LIT_MAX = 128;   // listed literals per clause; clauses with more are finished from their masks
constexpr int SP_WAVES = 16;   // wavefronts per workgroup of k_eval_sparse
constexpr int SP_PLANES = 8;   // bit planes of a wavefront's vote counter: at most 255 clauses per wavefront

// XB from row-major X: one workgroup of 4 wavefronts per 64 examples, each wavefront a
// contiguous share of the feature words; the 64 ballots of bit b of a word are two words
// of row 32 fw + b, their complement two words of row o + 32 fw + b.  Examples from q up
// to 32 QW read as feature 0 (no clause output is taken from them).  Row 2o is set to ones.
__global__ __launch_bounds__(256) void k_transpose_bits(const uint32_t *__restrict__ X, uint32_t *__restrict__ XB,
                                                        int64_t q, int Wf, int o, int QW)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + lane;
    if (threadIdx.x == 0) // this block's two words of the all-ones row
        *reinterpret_cast<uint2 *>(XB + (int64_t)2 * o * QW + (int64_t)blockIdx.x * 2) = make_uint2(~0u, ~0u);
    const int per = (Wf + 3) / 4;
    const int f_end = min(Wf, (wave + 1) * per);
    for (int fw = wave * per; fw < f_end; ++fw) {
        const uint32_t x = (i < q) ? X[i * Wf + fw] : 0u;
        uint64_t r = 0;
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            const uint64_t bal = ballot(((x >> b) & 1u) != 0u);
            r = (lane == b) ? bal : r;
        }
        const int k = fw * 32 + lane;
        if (lane < 32 && k < o) {
            *reinterpret_cast<uint2 *>(XB + (int64_t)k * QW + (int64_t)blockIdx.x * 2) =
                make_uint2((uint32_t)r, (uint32_t)(r >> 32));
            *reinterpret_cast<uint2 *>(XB + (int64_t)(o + k) * QW + (int64_t)blockIdx.x * 2) =
                make_uint2(~(uint32_t)r, ~(uint32_t)(r >> 32));
        }
    }
}

// Literal list of every clause, one wavefront per clause: entry = byte offset of the
// literal's row in XB; the first LIT_MAX included literals in literal order, the rest of
// the LIT_MAX slots filled with the all-ones row so that several clauses can be walked in
// step.  nlit[g] = number of included literals (may exceed LIT_MAX).
__global__ __launch_bounds__(256) void k_literal_lists(const uint32_t *__restrict__ inc, uint32_t *__restrict__ lits,
                                                       int32_t *__restrict__ nlit, int C, int Wf, int W, int o,
                                                       uint32_t row_bytes, int32_t *fresh, int qp)
{
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= C) return;
    // ahead of a tally pre-calculation: every stored output of the clause will be current
    if (fresh && lane == 0) *reinterpret_cast<int4 *>(fresh + (int64_t)g * 4) = make_int4(0, 0, qp, 0);
    uint32_t *L = lits + (int64_t)g * LIT_MAX;
    int base = 0;
    for (int w0 = 0; w0 < W; w0 += 64) {
        const int lw = w0 + lane;
        uint32_t m = lw < W ? inc[(int64_t)g * W + lw] : 0u;
        const int cnt = __builtin_popcount(m);
        int incl = cnt; // inclusive prefix sum over the lanes
#pragma unroll
        for (int dlt = 1; dlt < 64; dlt <<= 1) {
            const int t = __shfl_up(incl, dlt, 64);
            if (lane >= dlt) incl += t;
        }
        int pos = base + incl - cnt;
        const uint32_t k0 = lw >= Wf ? (uint32_t)o + (uint32_t)(lw - Wf) * 32u : (uint32_t)lw * 32u; // literal of bit 0
        while (m) {
            const int b = __builtin_ctz(m);
            m &= m - 1u;
            if (pos < LIT_MAX) L[pos] = (k0 + (uint32_t)b) * row_bytes;
            ++pos;
        }
        base += __shfl(incl, 63, 64);
    }
    for (int t = min(base, LIT_MAX) + lane; t < LIT_MAX; t += 64) L[t] = 2u * (uint32_t)o * row_bytes;
    if (lane == 0) nlit[g] = base;
}

struct SparseArgs {
    uint32_t *bits;      // [C][bits_stride] clause outputs, or null
    int64_t bits_stride;
    int32_t *acc;        // votes of class c for example i go to acc[i*acc_si + c*acc_sc], or null
    int64_t acc_si, acc_sc;
    int64_t q;
    int QW, QWq;         // words per row of XB; words that hold examples (ceil(q/32))
    int n, m, o, Wf, W;
    int ranges, by_xcd;  // ranges of 2048 examples; workgroup -> (range, class, share) mapping
    int S, chunk;        // clauses of a class are split over S workgroups, `chunk` (a multiple of 16) each
    int T;               // > 0: the sums are clamped to [-T, T] (only with S = 1)
};

// Output of clause g on the 32 examples of this lane's word, taken from its include masks
// (for the rare clause that has more than LIT_MAX literals and is still satisfied somewhere
// after the listed ones); `valid` masks examples >= q.
__device__ __forceinline__ uint32_t clause_from_masks(const uint32_t *__restrict__ inc, const char *xb_lane, int g,
                                                      uint32_t valid, const SparseArgs &a)
{
    uint32_t accv = valid;
    const uint32_t row_bytes = (uint32_t)a.QW * 4u;
    for (int lw = 0; lw < a.W; ++lw) {
        uint32_t m = inc[(int64_t)g * a.W + lw];
        const uint32_t k0 = lw >= a.Wf ? (uint32_t)a.o + (uint32_t)(lw - a.Wf) * 32u : (uint32_t)lw * 32u;
        while (m) {
            const int b = __builtin_ctz(m);
            m &= m - 1u;
            accv &= *reinterpret_cast<const uint32_t *>(xb_lane + (k0 + (uint32_t)b) * row_bytes);
        }
        if (ballot(accv != 0u) == 0) return 0u;
    }
    return accv;
}

// One workgroup per (range of 2048 examples, class c, share s of S).  It evaluates its share
// of the clauses of class c on the range: wavefront w takes the clauses j = j_lo + w + 16 k
// (all of one polarity, because j_lo and 16 are even), lane = word of 32 examples.
// Votes are counted bit-sliced: the outputs of eight clauses go through a tree of
// carry-save adders (two bit operations each) into ones/twos/fours and one ripple into
// the higher planes, about three operations per clause and word instead of one counter
// update per example.  At the end every wavefront adds its counts, signed by its
// polarity, into the workgroup's sums in LDS, and the workgroup writes them out: stored
// (and clamped when T > 0) if it holds all clauses of the class, added otherwise.
__global__ __launch_bounds__(64 * SP_WAVES) void k_eval_sparse(const uint32_t *__restrict__ lits,
                                                              const int32_t *__restrict__ nlit,
                                                              const uint32_t *__restrict__ inc,
                                                              const uint32_t *__restrict__ XB, const SparseArgs a)
{
    __shared__ int32_t sums[64 * 33]; // [word of the range][example of the word], rows padded against bank conflicts
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups go to the 8 XCDs in turn and every XCD has its own L2.  With many ranges
    // XCD x is given the ranges x, x + 8, ...: then only an eighth of every literal row
    // passes through each L2 (same speed, a third of the HBM fetches).
    int range = blockIdx.x, cs = blockIdx.y;
    if (a.by_xcd) {
        const int mS = a.m * a.S;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        range = xcd + 8 * (slot / mS);
        cs = slot - (slot / mS) * mS;
        if (range >= a.ranges) return;
    }
    const int c = cs / a.S, s = cs - c * a.S;
    const int word0 = range * 64, word = word0 + lane;
    uint32_t valid = 0u;
    if (word < a.QWq) {
        const int64_t rem = a.q - (int64_t)word * 32;
        valid = rem >= 32 ? ~0u : ((1u << (int)rem) - 1u);
    }
    const char *xb_lane = reinterpret_cast<const char *>(XB + word);
    const char *xb_base = reinterpret_cast<const char *>(XB);
    uint32_t word_off = (uint32_t)word * 4u;
    asm volatile("" : "+v"(word_off)); // keep the sum in the vector unit
    if (a.acc) {
        for (int t = tid; t < 64 * 33; t += 64 * SP_WAVES) sums[t] = 0;
        __syncthreads();
    }
    uint32_t planes[SP_PLANES];
#pragma unroll
    for (int pl = 0; pl < SP_PLANES; ++pl) planes[pl] = 0u;
    const int j_lo = s * a.chunk, j_hi = min(a.n, j_lo + a.chunk);
    auto csa = [](uint32_t &hi, uint32_t &lo, uint32_t x, uint32_t y, uint32_t z) {
        hi = majority3(x, y, z);
        lo = xor3(x, y, z);
    };
    for (int j0 = j_lo + wave; j0 < j_hi; j0 += 8 * SP_WAVES) {
        // eight clauses are walked in step, four literals each per round: 32 loads in flight
        uint32_t x[8];
        const uint32_t *L[8];
        int nl[8], longest = 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u * SP_WAVES;
            const bool ok = j < j_hi;
            const int g = c * a.n + (ok ? j : j_lo);
            L[u] = lits + (int64_t)g * LIT_MAX;
            nl[u] = ok ? nlit[g] : 0;
            x[u] = ok ? valid : 0u;
            longest = max(longest, min(nl[u], LIT_MAX));
        }
        for (int k = 0; k < longest; k += 4) {
            uint32_t r[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                // past a list's end: the all-ones row.  Row offset (uniform) + word offset (per lane)
                // are added in the vector unit: one operation instead of a 64-bit scalar add per
                // load.  (Buffer loads that take the row offset as their scalar offset need no add
                // at all, but measured 45 % slower: the list entries then sit in scalar registers
                // until their load is issued, and too few list loads stay in flight.)
                const uint4 e = *reinterpret_cast<const uint4 *>(L[u] + k);
                r[u][0] = *reinterpret_cast<const uint32_t *>(xb_base + (e.x + word_off));
                r[u][1] = *reinterpret_cast<const uint32_t *>(xb_base + (e.y + word_off));
                r[u][2] = *reinterpret_cast<const uint32_t *>(xb_base + (e.z + word_off));
                r[u][3] = *reinterpret_cast<const uint32_t *>(xb_base + (e.w + word_off));
            }
            uint32_t any = 0u;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x[u] &= r[u][0] & r[u][1] & r[u][2] & r[u][3];
                any |= x[u];
            }
            if (ballot(any != 0u) == 0) break; // every clause has a false literal on every example of the range
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u * SP_WAVES;
            if (j < j_hi) {
                const int g = c * a.n + j;
                if (nl[u] > LIT_MAX && ballot(x[u] != 0u) != 0) x[u] = clause_from_masks(inc, xb_lane, g, valid, a);
                if (a.bits && word < a.bits_stride) a.bits[(int64_t)g * a.bits_stride + word] = x[u];
            }
        }
        if (a.acc) {
            uint32_t t2a, t2b, t4a, t4b, e8;
            csa(t2a, planes[0], planes[0], x[0], x[1]);
            csa(t2b, planes[0], planes[0], x[2], x[3]);
            csa(t4a, planes[1], planes[1], t2a, t2b);
            csa(t2a, planes[0], planes[0], x[4], x[5]);
            csa(t2b, planes[0], planes[0], x[6], x[7]);
            csa(t4b, planes[1], planes[1], t2a, t2b);
            csa(e8, planes[2], planes[2], t4a, t4b);
#pragma unroll
            for (int pl = 3; pl < SP_PLANES; ++pl) { // ripple the carry of weight 8 upwards
                const uint32_t t = planes[pl] & e8;
                planes[pl] ^= e8;
                e8 = t;
            }
        }
    }
    if (!a.acc) return;
    const bool positive = (wave & 1) != 0; // odd index within the class: positive polarity
#pragma unroll 4
    for (int e = 0; e < 32; ++e) {
        int v = 0;
#pragma unroll
        for (int pl = 0; pl < SP_PLANES; ++pl) v |= (int)((planes[pl] >> e) & 1u) << pl;
        if (v) atomicAdd(&sums[lane * 33 + e], positive ? v : -v);
    }
    __syncthreads();
    for (int idx = tid; idx < 2048; idx += 64 * SP_WAVES) {
        const int64_t i = (int64_t)word0 * 32 + idx;
        if (i >= a.q) continue;
        int v = sums[(idx >> 5) * 33 + (idx & 31)];
        int32_t *dst = a.acc + i * a.acc_si + (int64_t)c * a.acc_sc;
        if (a.S == 1) *dst = a.T > 0 ? min(max(v, -a.T), a.T) : v;
        else if (v) atomicAdd(dst, v);
    }
}

// ------------------------------------------------------------------------
// k_train: Algorithm 1, one wavefront per clause
// ------------------------------------------------------------------------

struct TrainArgs {
    Dims d;
    SatConst sat;
    uint32_t *planes;
    uint32_t *inc;
    int32_t *tally;
    const int32_t *vhat; // [q][m] snapshot the gate reads instead of the live tally, or null
    uint32_t *ostar;
    int32_t *fresh; // [C][4] per clause: examples whose stored output may be outdated lie in [plo,phi) or [slo,qp)
    const int32_t *order; // [C] clause handled by each wavefront of the launch
    unsigned long long *counters;
    int32_t q, qp, Qw, i_begin, i_end; // example counts fit 31 bits (checked at bind)
    uint32_t epoch;
    int lds_mask_words; // W rounded up to a multiple of 4
    int lds_off_words;  // Wf + EVAL_PAD rounded up to a multiple of 4
    int lds_wave_words; // LDS words per wavefront
    int QW;             // words per row of XB
};

constexpr int EVAL_PAD = 16; // empty entries after the list: a group may read that far past its end

// The clause as the evaluation loop wants it: one entry per feature word whose
// plain or negated mask word is non-zero, compacted in LDS: eoff[k] = byte
// offset of that word's row in XT, emask[k] = {mask of plain literals, mask of
// negated literals}; padded with EVAL_PAD empty entries.  Rebuilt whenever plane 7
// changes.
template <int WPL>
__device__ __forceinline__ int build_entries(const u32x8 (&p)[WPL], uint32_t *lmask, uint32_t *eoff,
                                             uint2 *emask, int lane, int Wf, int W, uint32_t row_bytes)
{
#pragma unroll
    for (int r = 0; r < WPL; ++r) {
        const int lw = r * 64 + lane;
        if (lw < W) lmask[lw] = p[r][7];
    }
    wave_lds_sync();
    int n = 0;
    for (int f0 = 0; f0 < Wf; f0 += 64) {
        const int fw = f0 + lane;
        const bool ok = fw < Wf;
        const uint32_t mp = ok ? lmask[fw] : 0u;
        const uint32_t mn = ok ? lmask[Wf + fw] : 0u;
        const bool nzf = (mp | mn) != 0u;
        const uint64_t b = ballot(nzf);
        const int pre = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u));
        if (nzf) {
            eoff[n + pre] = (uint32_t)fw * row_bytes;
            emask[n + pre] = make_uint2(mp, mn);
        }
        n += __builtin_popcountll(b);
    }
    if (lane < EVAL_PAD) {
        eoff[n + lane] = 0u;
        emask[n + lane] = make_uint2(0u, 0u);
    }
    wave_lds_sync();
    return n;
}

// Clause outputs for 64 examples, lane = example: bit l of the result is
// C(X_{i0+l}).  xt_block points at XT[0][i0].  An entry costs one coalesced
// 256-byte load, an LDS broadcast of its masks and two bit operations.
// Entries are taken EVAL_GROUP at a time (that many loads in flight; 8 and 24
// measured slower); a dense (young) clause violates all 64 examples within the
// first group and the loop stops.
constexpr int EVAL_GROUP = 16;

__device__ __forceinline__ uint64_t eval64(const uint32_t *eoff, const uint2 *emask, int nent,
                                           const uint32_t *__restrict__ xt_block, int lane)
{
    uint32_t viol = 0;
    const char *base = reinterpret_cast<const char *>(xt_block);
    const uint32_t lane4 = (uint32_t)lane * 4u;
    for (int k = 0; k < nent; k += EVAL_GROUP) {
        uint32_t off[EVAL_GROUP], x[EVAL_GROUP];
#pragma unroll
        for (int j = 0; j < EVAL_GROUP; j += 4) {
            const uint4 o = *reinterpret_cast<const uint4 *>(eoff + k + j);
            off[j] = o.x; off[j + 1] = o.y; off[j + 2] = o.z; off[j + 3] = o.w;
        }
#pragma unroll
        for (int j = 0; j < EVAL_GROUP; ++j) x[j] = *reinterpret_cast<const uint32_t *>(base + (off[j] + lane4));
        const uint4 *mq = reinterpret_cast<const uint4 *>(emask + k);
#pragma unroll
        for (int j = 0; j < EVAL_GROUP / 2; ++j) {
            const uint4 m = mq[j]; // {plain, negated} masks of entries 2j and 2j+1
            // a plain literal is violated where x = 0, a negated one where x = 1
            viol |= bitselect(x[2 * j], m.y, m.x) | bitselect(x[2 * j + 1], m.w, m.z);
        }
        if (ballot(viol == 0u) == 0) break;
    }
    return ballot(viol == 0u);
}

// Literals a clause's list in LDS can hold for the sweeps over outdated outputs; clauses
// with more (untrained ones) are swept block by block with eval64.
constexpr int TRAIN_LIT_MAX = 64;

// Number of included literals of the clause held in p: the per-lane counts are summed bit by
// bit with ballots, a loop-free wave sum.  (An atomic add on one LDS word would do, but the
// compiler expands it into a 64-step scalar loop over the lanes.)
template <int WPL>
__device__ __forceinline__ int count_literals(const u32x8 (&p)[WPL], int lane, int W)
{
    uint32_t cnt = 0;
#pragma unroll
    for (int r = 0; r < WPL; ++r) cnt += (r * 64 + lane < W) ? (uint32_t)__builtin_popcount(p[r][7]) : 0u;
    int total = 0;
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) // cnt <= 32 * WPL <= 128 for the narrow clauses this is used for
        total += __builtin_popcountll(ballot(((cnt >> bit) & 1u) != 0u)) << bit;
    return total;
}

// List of the included literals of the clause held in p (lane = literal word), as byte
// offsets of their rows in XB, padded to a multiple of 4 with the all-ones row; returns
// the number of included literals.  Only called for clauses with at most TRAIN_LIT_MAX.
// The order of the list does not matter (the output is their conjunction): literals are
// taken bit position by bit position, each position compacted over the lanes by ballot.
template <int WPL>
__device__ __forceinline__ int build_literals(const u32x8 (&p)[WPL], uint32_t *llist, int lane, int Wf, int W, int o,
                                              uint32_t xb_row_bytes)
{
    int base = 0;
#pragma unroll
    for (int r = 0; r < WPL; ++r) {
        const int lw = r * 64 + lane;
        const uint32_t m = lw < W ? p[r][7] : 0u;
        if (ballot(m != 0u) == 0) continue;
        const uint32_t k0 = lw >= Wf ? (uint32_t)o + (uint32_t)(lw - Wf) * 32u : (uint32_t)lw * 32u; // literal of bit 0
        for (int b = 0; b < 32; ++b) {
            const bool set = ((m >> b) & 1u) != 0u;
            const uint64_t bal = ballot(set);
            if (bal == 0) continue;
            const int pos = base + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            if (set && pos < TRAIN_LIT_MAX) llist[pos] = (k0 + (uint32_t)b) * xb_row_bytes;
            base += __builtin_popcountll(bal);
        }
    }
    if (lane < 4) llist[min(base, TRAIN_LIT_MAX) + lane] = 2u * (uint32_t)o * xb_row_bytes;
    wave_lds_sync();
    return base;
}

constexpr int TRAIN_WAVES = 4; // clauses (wavefronts) per workgroup of the training kernel

// One wavefront = one clause of class c.  The examples whose gate can open for this
// clause are those of the gate list of c for this launch (label c: trained towards 1;
// drawn negative class c: trained towards 0); their gates are drawn 64 at a time, lane =
// list entry.  Blocks of 64 consecutive examples are evaluated (lane = example) only
// when a gate in them fired or their stored outputs may be outdated; all other blocks
// of the pass are never touched.
template <int WPL, bool FULL>
__global__ __launch_bounds__(64 * TRAIN_WAVES) void k_train(const uint32_t *__restrict__ X, const uint32_t *__restrict__ XT,
                                                            const uint32_t *__restrict__ XB,
                                                            const int32_t *__restrict__ gate,
                                                            const int32_t *__restrict__ ngate, const TrainArgs a)
{
    extern __shared__ uint32_t lds[];
    const Dims &d = a.d;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int slot = blockIdx.x * TRAIN_WAVES + wave;
    if (slot >= d.C) return; // whole wavefront; the kernel has no workgroup-wide barrier
    const int g = __builtin_amdgcn_readfirstlane(a.order[slot]);
    uint32_t *lmask = lds + wave * a.lds_wave_words;        // [W] include masks, literal-word order
    uint32_t *eoff = lmask + a.lds_mask_words;              // [Wf + EVAL_PAD] (rounded to 4 words)
    uint2 *emask = reinterpret_cast<uint2 *>(eoff + a.lds_off_words);
    uint32_t *llist = lmask + a.lds_wave_words - (TRAIN_LIT_MAX + 4); // [TRAIN_LIT_MAX + 4] literal list for the sweeps

    const int c = g / d.n;
    const bool pos = ((g - c * d.n) & 1) != 0; // odd index within the class: positive polarity
    const int sign = pos ? 1 : -1;
    const int T = d.T;
    const uint32_t row_bytes = (uint32_t)a.qp * 4u;
    const int i_begin = a.i_begin, i_end = a.i_end, q = a.q;

    u32x8 p[WPL];
#pragma unroll
    for (int r = 0; r < WPL; ++r) {
        const int lw = r * 64 + lane;
        u32x8 t = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        if (lw < d.W) {
            const uint4 *src = reinterpret_cast<const uint4 *>(a.planes + ((int64_t)g * d.W + lw) * 8);
            const uint4 v0 = src[0], v1 = src[1];
            t[0] = v0.x; t[1] = v0.y; t[2] = v0.z; t[3] = v0.w;
            t[4] = v1.x; t[5] = v1.y; t[6] = v1.z; t[7] = v1.w;
        }
        p[r] = t;
    }
    int nent = build_entries<WPL>(p, lmask, eoff, emask, lane, d.Wf, d.W, row_bytes);

    // lowest Philox block of the Type I comparator that can matter: bits of the
    // uniform below the lowest set bit of thr never decide u < thr
    const int tz = d.thr ? __builtin_ctz(d.thr) : 16;
    const int first_blk = min(tz >> 2, 4);
    const uint32_t ge_init = d.thr >= 65536u ? 0u : ~0u;

    // per-wavefront event counts of one launch fit 32 bits (at most 2^30 examples per launch)
    uint32_t n_fired = 0, n_type1 = 0, n_changes = 0, n_type2 = 0, n_eval = 0, n_draw = 0, n_listed_blocks = 0;

    // Which stored previous outputs o* can differ from the clause's current output: only
    // those not re-evaluated since the include mask last changed.  Kept per clause as two
    // example ranges (multiples of 64), a prefix part [plo, phi) and a suffix [slo, qp); a
    // block outside both needs no evaluation and no refresh unless one of its gates fires
    // (the result is the same as refreshing every visited pair: o != o* would be false).
    int plo, phi, slo;
    {
        const int4 f = *reinterpret_cast<const int4 *>(a.fresh + (int64_t)g * 4);
        plo = __builtin_amdgcn_readfirstlane(f.x);
        phi = __builtin_amdgcn_readfirstlane(f.y);
        slo = __builtin_amdgcn_readfirstlane(f.z);
    }
    auto next_stale = [&](int b) { // first block index >= b that may hold outdated outputs
        int r = max(b, slo >> 6);
        if (plo < phi && b < ((phi + 63) >> 6)) r = min(r, max(b, plo >> 6));
        return r;
    };

    // the gate list of this class for this launch
    const int32_t *list = gate + (int64_t)c * a.qp;
    const int k_lo = 0, k_hi = ngate[c];
    const int32_t *tally_c = a.tally + (int64_t)c * a.qp;

    // state of the block of 64 examples that is currently open (cb < 0: none)
    const int end_block = (i_end + 63) >> 6;
    int cb = -1, next_block = i_begin >> 6;
    uint64_t obits = 0, ost = 0, rmask = 0;
    bool mask_changed = false;

    auto range_mask = [&](int b0) { return ballot(b0 + lane >= i_begin && b0 + lane < i_end); };
    auto pack64 = [&](uint32_t lo, uint32_t hi) {
        return (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)lo) |
               ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)hi) << 32);
    };
    // Refresh of tally and previous-output bits (last lines of Algorithm 1) for the 64
    // examples of block b at once: ob = outputs with the current masks, os = stored ones,
    // rm = examples of the block that belong to this launch.
    auto refresh_block = [&](int b, uint64_t ob, uint64_t os, uint64_t rm) {
        const int b0 = b << 6;
        const uint64_t diff = (ob ^ os) & rm;
        if (diff) {
            if ((diff >> lane) & 1ull) {
                const int delta = ((ob >> lane) & 1ull) ? sign : -sign;
                atomicAdd(&a.tally[(int64_t)c * a.qp + b0 + lane], delta);
            }
            const uint64_t nw = os ^ diff;
            if (lane == 0) {
                uint32_t *op = a.ostar + (int64_t)g * a.Qw + (b0 >> 5);
                op[0] = (uint32_t)nw;
                op[1] = (uint32_t)(nw >> 32);
            }
            n_changes += __builtin_popcountll(diff);
        }
    };
    // ... followed by the bookkeeping of which stored outputs may be outdated
    auto close_block = [&](int b, uint64_t ob, uint64_t os, uint64_t rm, bool changed) {
        refresh_block(b, ob, os, rm);
        const int b0 = b << 6, b1 = b0 + 64;
        const bool whole = b0 >= i_begin && (b1 <= i_end || i_end == q);
        if (whole) { // this block is up to date again
            if (b0 <= plo) plo = max(plo, b1);
            if (b0 <= slo) slo = max(slo, b1);
        }
        if (changed) { // everything not visited after the change is outdated now
            plo = 0;
            phi = b1;
            slo = b1;
        }
    };
    // Refresh of every block in [from, to) that may hold outdated outputs; no gate fired in
    // them, so the masks stay as they are.  After a mask change these are all the blocks up
    // to the next fired gate, most of what an epoch of a trained machine has to evaluate.
    // A trained clause has few literals, so the sweep walks its literal list over the rows
    // of XB, lane = word of 32 examples: 2048 examples per pass and one load per literal.
    int n_listed = -1;          // literals of the current masks (list built if <= TRAIN_LIT_MAX), -1: not counted since the last change
    uint32_t n_changes_v = 0;   // tally changes found by the passes, per lane
    const char *xb_base = reinterpret_cast<const char *>(XB);
    uint32_t *ostar_row = a.ostar + (int64_t)g * a.Qw;
    auto sweep_listed = [&](int bs, int be) { // blocks [bs, be), all of them possibly outdated
        for (int w0 = 2 * bs; w0 < 2 * be; w0 += 64) {
            const int w = w0 + lane;
            const bool act = w < 2 * be;
            const int e0 = w << 5;
            const int lo = min(max(i_begin - e0, 0), 32), hi = min(max(i_end - e0, 0), 32);
            uint32_t rm = 0u; // examples of the word that belong to this launch
            if (act && hi > lo) rm = (hi == 32 ? ~0u : (1u << hi) - 1u) & ~((1u << lo) - 1u);
            const uint32_t woff = act ? (uint32_t)w * 4u : 0u;
            const uint32_t ost = act ? ostar_row[w] : 0u;
            uint32_t accv = rm;
            for (int k = 0; k < n_listed; k += 4) {
                const uint4 e = *reinterpret_cast<const uint4 *>(llist + k);
                const uint32_t x0 = *reinterpret_cast<const uint32_t *>(xb_base + (e.x + woff));
                const uint32_t x1 = *reinterpret_cast<const uint32_t *>(xb_base + (e.y + woff));
                const uint32_t x2 = *reinterpret_cast<const uint32_t *>(xb_base + (e.z + woff));
                const uint32_t x3 = *reinterpret_cast<const uint32_t *>(xb_base + (e.w + woff));
                accv &= x0 & x1 & x2 & x3;
            }
            uint32_t diff = (accv ^ ost) & rm;
            if (diff) ostar_row[w] = ost ^ diff;
            n_changes_v += (uint32_t)__builtin_popcount(diff);
            while (diff) { // one tally correction per changed example
                const int bit = __builtin_ctz(diff);
                diff &= diff - 1u;
                atomicAdd(&a.tally[(int64_t)c * a.qp + e0 + bit], ((accv >> bit) & 1u) ? sign : -sign);
            }
        }
        n_eval += (uint32_t)(be - bs);
        n_listed_blocks += (uint32_t)(be - bs);
        // the whole blocks among them are up to date again
        const int fs = max(bs, (i_begin + 63) >> 6), fe = (i_end == q) ? be : min(be, i_end >> 6);
        if (fs < fe) {
            const int b0 = fs << 6, b1 = fe << 6;
            if (b0 <= plo) plo = max(plo, b1);
            if (b0 <= slo) slo = max(slo, b1);
        }
    };
    auto sweep = [&](int from, int to) {
        if (next_stale(from) >= to) return;
        // the outdated blocks are those of [plo, phi) and of [slo, qp), in this order
        int s1 = from, e1 = from;
        if (plo < phi) {
            s1 = max(from, plo >> 6);
            e1 = max(s1, min(to, (phi + 63) >> 6));
        }
        const int s2 = max(max(from, slo >> 6), e1);
        const int n_blocks = (e1 - s1) + max(to - s2, 0);
        // The list pays for runs of blocks: a few blocks, or a list that the last mask change
        // left to be rebuilt for a short run, are cheaper block by block below; so are wide
        // clauses (their registers hold the automata) and untrained ones (hundreds of literals).
        if (WPL <= 4 && n_blocks >= (n_listed < 0 ? 8 : 3)) {
            if (n_listed < 0) {
                n_listed = count_literals<WPL>(p, lane, d.W);
                if (n_listed <= TRAIN_LIT_MAX) build_literals<WPL>(p, llist, lane, d.Wf, d.W, d.o, (uint32_t)a.QW * 4u);
            }
            if (n_listed <= TRAIN_LIT_MAX) {
                if (s1 < e1) sweep_listed(s1, e1);
                if (s2 < to) sweep_listed(s2, to);
                return;
            }
        }
        for (int b = next_stale(from); b < to; b = next_stale(b + 1)) { // closing b does not change which later blocks are outdated
            const uint32_t *op = ostar_row + (b << 1);
            const uint32_t o0 = op[0], o1 = op[1];
            const uint64_t ob = eval64(eoff, emask, nent, XT + (b << 6), lane);
            close_block(b, ob, pack64(o0, o1), range_mask(b << 6), false);
            ++n_eval;
        }
    };

    // Candidate data are fetched ahead: entry words two candidate blocks ahead, tallies (which
    // need the entry's example index) one block ahead.  Reading a tally early is within the
    // method's premise of outdated tallies.
    auto load_ent = [&](int k0) { // packed (example << 1 | target), or -1 beyond the range
        const int k = k0 + lane;
        return k < k_hi ? list[k] : -1;
    };
    auto load_v = [&](int ent) {
        if (ent < 0) return 0;
        const int i = ent >> 1;
        return a.vhat ? a.vhat[(int64_t)i * d.m + c]
                      : __hip_atomic_load(&tally_c[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    int ent_cur = load_ent(k_lo);
    int v_cur = load_v(ent_cur);
    int ent_nxt = load_ent(k_lo + 64);

    for (int k0 = k_lo;; k0 += 64) {
        const bool last = k0 >= k_hi; // all candidates done: one more round sweeps the remaining blocks
        uint64_t fmask = 0, tmask = 0;
        int iv = 0;
        if (!last) {
            const int ent = ent_cur, v = v_cur;
            ent_cur = ent_nxt;
            v_cur = load_v(ent_cur);
            ent_nxt = load_ent(k0 + 128);
            const bool valid = ent >= 0;
            iv = ent >> 1;
            const bool target = (ent & 1) != 0;
            bool fire = false, open = false;
            if (valid) {
                const int vc = min(max(v, -T), T);
                const int e = target ? T - vc : T + vc; // Algorithm 1: error of the recorded vote sum
                open = e > 0;
                if (open) {
                    const U4 r = draw(d.key, STREAM_GATE, 0, (uint32_t)g, (uint64_t)(uint32_t)iv, a.epoch);
                    fire = (uint64_t)r.x * (uint64_t)(2 * (int64_t)T) < ((uint64_t)e << 32);
                }
            }
            fmask = ballot(fire);
            tmask = ballot(target);
            n_draw += __builtin_popcountll(ballot(open));
            n_fired += __builtin_popcountll(fmask);
        }

        // words of a fired example in lane = literal-word layout.  Slot geometry (which half,
        // which bits exist) is recomputed from a laundered index wherever it is needed: it is
        // example-independent, and the compiler would otherwise keep it in VGPRs for every slot.
        auto load_row = [&](int ii, uint32_t (&dst)[WPL]) {
            const uint32_t *xrow = X + (int64_t)ii * d.Wf;
#pragma unroll
            for (int r = 0; r < WPL; ++r) {
                uint32_t lw = (uint32_t)(r * 64 + lane);
                asm volatile("" : "+v"(lw));
                const bool act = lw < (uint32_t)d.W;
                const uint32_t fw = act ? (lw >= (uint32_t)d.Wf ? lw - (uint32_t)d.Wf : lw) : 0u;
                dst[r] = xrow[fw];
            }
        };
        // the row of the next fired example is requested while the current one is processed
        uint32_t xnext[WPL];
        if (fmask) load_row(__builtin_amdgcn_readlane(iv, __builtin_ctzll(fmask)), xnext);

        for (;;) {
            // next event: a fired candidate, or (after the last candidate) the end of the range
            const bool have = fmask != 0;
            int l = 0, ii = 0, B;
            if (have) {
                l = __builtin_ctzll(fmask);
                fmask &= fmask - 1;
                ii = __builtin_amdgcn_readlane(iv, l);
                B = ii >> 6;
            } else if (last) {
                B = end_block;
            } else {
                break;
            }

            // bring block B up: close the open block, refresh the outdated blocks in between
            if (cb != B) {
                if (cb >= 0) {
                    close_block(cb, obits, ost, rmask, mask_changed);
                    next_block = cb + 1;
                    cb = -1;
                }
                const int lim = min(B, end_block);
                sweep(next_block, lim);
                next_block = max(next_block, lim);
                if (B < end_block) {
                    // open block B: previous outputs, range mask, evaluation with the current masks
                    cb = B;
                    const int b0 = B << 6;
                    const uint32_t *op = a.ostar + (int64_t)g * a.Qw + (b0 >> 5);
                    const uint32_t o0 = op[0], o1 = op[1];
                    rmask = range_mask(b0);
                    obits = eval64(eoff, emask, nent, XT + b0, lane);
                    ost = pack64(o0, o1);
                    mask_changed = false;
                    ++n_eval;
                }
            }
            if (!have) break; // the range is finished

            const int bl = ii & 63;                  // position of the example in the open block
            const bool tgt = (tmask >> l) & 1;
            const bool Cout = (obits >> bl) & 1;     // clause output on the state before the update
            uint32_t changed = 0;
            uint32_t xw[WPL];
#pragma unroll
            for (int r = 0; r < WPL; ++r) xw[r] = xnext[r];
            if (fmask) load_row(__builtin_amdgcn_readlane(iv, __builtin_ctzll(fmask)), xnext);
            auto literal = [&](uint32_t lw, uint32_t x, uint32_t &valid) {
                const bool act = lw < (uint32_t)d.W;
                const bool neg = lw >= (uint32_t)d.Wf;
                const uint32_t fw = neg ? lw - (uint32_t)d.Wf : lw;
                valid = act ? (fw == (uint32_t)d.Wf - 1u ? d.tailmask : ~0u) : 0u;
                return (x ^ (neg ? ~0u : 0u)) & valid; // 0 on padding bits and idle lanes
            };
            if (tgt != pos) {
                // Type II feedback (Table 2): where the clause is 1 and the literal 0, push Exclude towards Include
                if (Cout) {
                    ++n_type2;
#pragma unroll
                    for (int r = 0; r < WPL; ++r) {
                        uint32_t lw = (uint32_t)(r * 64 + lane);
                        asm volatile("" : "+v"(lw));
                        uint32_t valid;
                        const uint32_t lit = literal(lw, xw[r], valid);
                        uint32_t sp[8];
                        get_slot(p[r], sp);
                        const uint32_t old7 = sp[7];
                        const uint32_t m = ~lit & ~old7 & valid; // excluded automata (below the top bit) cannot overflow
                        ripple_inc(sp, m);
                        changed |= sp[7] ^ old7;
                        put_slot(p[r], sp);
                    }
                }
            } else {
                // Type I feedback (Table 1)
                ++n_type1;
#pragma unroll
                for (int r = 0; r < WPL; ++r) {
                    // The literal-word index is laundered through an empty asm so that the
                    // compiler does not hoist the example-independent first Philox round of
                    // every slot and block out of the example loop (dozens of live VGPRs per slot).
                    uint32_t lw = (uint32_t)(r * 64 + lane);
                    asm volatile("" : "+v"(lw));
                    // bit-sliced comparison of 32 16-bit uniforms with thr, least significant bit first:
                    // ge = [u >= thr]; bit b of literal j's uniform is bit j of random word b;
                    // thr bit 1: ge &= w, thr bit 0: ge |= w, i.e. majority(w, ge, ~thr bit)
                    uint32_t ge = ge_init;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        if (t >= first_blk) {
                            const U4 R = draw(d.key, STREAM_TYPE1, 4u * lw + (uint32_t)t, (uint32_t)g,
                                              (uint64_t)(uint32_t)ii, a.epoch);
                            const uint32_t w[4] = {R.x, R.y, R.z, R.w};
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const uint32_t K = ((d.thr >> (4 * t + k)) & 1u) ? 0u : ~0u;
                                ge = majority3(w[k], ge, K);
                            }
                        }
                    }
                    uint32_t valid;
                    const uint32_t lit = literal(lw, xw[r], valid);
                    uint32_t sp[8];
                    get_slot(p[r], sp);
                    const uint32_t old7 = sp[7];
                    if (Cout) { // strong: literals that are 1 move towards Include with probability (s-1)/s (1 if boosted)
                        const uint32_t m = lit & (ge | d.boost) & ~at_value<FULL>(sp, a.sat.kmax, true);
                        ripple_inc(sp, m);
                    }
                    // weak: everything else moves towards Exclude with probability 1/s
                    const uint32_t wk = (Cout ? ~lit : ~0u) & ~ge & valid & ~at_value<FULL>(sp, a.sat.kmin, false);
                    ripple_dec(sp, wk);
                    changed |= sp[7] ^ old7;
                    put_slot(p[r], sp);
                    // keep the slots apart in the instruction schedule: interleaving them
                    // multiplies the live registers by the number of slots
                    if (WPL > 2) __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (ballot(changed != 0u)) { // the conjunction changed: re-evaluate this and the later examples of the block
                mask_changed = true;
                n_listed = -1;
                nent = build_entries<WPL>(p, lmask, eoff, emask, lane, d.Wf, d.W, row_bytes);
                const uint64_t nb = eval64(eoff, emask, nent, XT + (cb << 6), lane);
                const uint64_t keep = (1ull << bl) - 1ull;
                obits = (obits & keep) | (nb & ~keep);
            }
        }
        if (last) break;
    }
    if (plo >= phi) plo = phi = 0;
    if (lane == 0) *reinterpret_cast<int4 *>(a.fresh + (int64_t)g * 4) = make_int4(plo, phi, slo, 0);

#pragma unroll
    for (int r = 0; r < WPL; ++r) {
        const int lw = r * 64 + lane;
        if (lw < d.W) {
            uint4 *dst = reinterpret_cast<uint4 *>(a.planes + ((int64_t)g * d.W + lw) * 8);
            const u32x8 t = p[r];
            dst[0] = make_uint4(t[0], t[1], t[2], t[3]);
            dst[1] = make_uint4(t[4], t[5], t[6], t[7]);
            a.inc[(int64_t)g * d.W + lw] = t[7];
        }
    }
    for (int sh = 32; sh > 0; sh >>= 1) n_changes_v += __shfl_xor(n_changes_v, sh, 64);
    n_changes += n_changes_v;
    // event counters: 64 interleaved sets, because thousands of wavefronts ending at the
    // same time on one address serialise in the L2 atomic unit (measured: ~1.7 ms per launch)
    if (lane < 8) { // slot 4 (trained pairs) is counted by the launch preparation
        const uint32_t v = lane == 0 ? n_listed_blocks : lane == 1 ? n_fired : lane == 2 ? n_type1 : lane == 3 ? n_changes
                         : lane == 4 ? 0u : lane == 5 ? n_type2 : lane == 6 ? n_eval : n_draw;
        if (v) atomicAdd(&a.counters[(g & (COUNTER_SETS - 1)) * 8 + lane], (unsigned long long)v);
    }
}

} // namespace tsetlin

// ------------------------------------------------------------------------
// host side: handle, validation, launches
// ------------------------------------------------------------------------

using namespace tsetlin;

struct tm_handle {
    tm_config cfg;
    Dims d;
    SatConst sat;
    uint32_t *planes;
    uint32_t *inc;
    // bound training data
    bool bound;
    const uint32_t *X;
    const int32_t *y;
    int64_t q, qp, Qw;
    int32_t *tally;
    uint32_t *ostar;
    uint32_t *XT;
    int32_t *negcls;
    uint32_t *XB;   // [2o+1][QW] literal rows of the bound data
    uint32_t *lits; // [C][LIT_MAX]
    int32_t *nlit;  // [C]
    int32_t *gate;  // [m][qp] gate lists of the current launch
    int32_t *ngate; // [m]
    int32_t *fresh;
    int32_t *order; // [C] launch order of the clauses
    int32_t *seg_cnt; // [m + 1][segments][2] flagged items per segment of the launch preparation
    unsigned long long *counters;
    int32_t *flag;
    uint32_t epoch;
    uint64_t pairs_visited; // (clause, example) visits enqueued since the counters were last read
    int last_hip;
    // kernel timing (measurement aid): event pairs around the launches of the two main kernels
    bool timing;
    std::vector<hipEvent_t> ev_pool;  // events created so far, reused
    size_t ev_used;                   // events of the pool handed out since timing was switched on
    std::vector<int> ev_kind;         // kind of the k-th recorded pair (events 2k, 2k+1)
};

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int check_config(const tm_config *cfg)
{
    if (!cfg) return TM_EINVAL;
    if (cfg->n_classes < 2 || cfg->clauses_per_class < 2 || (cfg->clauses_per_class & 1)) return TM_EINVAL;
    if (cfg->n_features < 1) return TM_EINVAL;
    if (cfg->states_per_action < 1 || cfg->states_per_action > 128) return TM_EINVAL;
    if (cfg->T < 1 || cfg->T > (1 << 29)) return TM_EINVAL;
    if (!(cfg->s >= 1.0) || !isfinite(cfg->s)) return TM_EINVAL;
    if (cfg->device < 0) return TM_EINVAL;
    if (cfg->boost_true_positive != 0 && cfg->boost_true_positive != 1) return TM_EINVAL;
    if (cfg->n_features > TM_MAX_FEATURES) return TM_ELIMIT;
    if ((int64_t)cfg->n_classes * cfg->clauses_per_class > (int64_t)1 << 30) return TM_ELIMIT;
    return TM_OK;
}

Dims make_dims(const tm_config *cfg)
{
    Dims d;
    d.m = cfg->n_classes;
    d.n = cfg->clauses_per_class;
    d.o = cfg->n_features;
    d.N = cfg->states_per_action;
    d.T = cfg->T;
    d.C = d.m * d.n;
    d.Wf = (d.o + 31) / 32;
    d.W = 2 * d.Wf;
    double t = floor(65536.0 / cfg->s + 0.5); // P(u < thr) = 1/s at 16-bit resolution
    if (t < 0.0) t = 0.0;
    if (t > 65536.0) t = 65536.0;
    d.thr = (uint32_t)t;
    d.boost = cfg->boost_true_positive ? ~0u : 0u;
    d.tailmask = (d.o & 31) ? ((1u << (d.o & 31)) - 1u) : ~0u;
    d.key.seed_lo = (uint32_t)(cfg->seed & 0xffffffffu);
    d.key.seed_hi = (uint32_t)(cfg->seed >> 32);
    return d;
}

// words per row of XB for q examples: whole ranges of 2048 examples
inline int64_t xb_row_words(int64_t q) { return ((q + 2047) / 2048) * 64; }
inline size_t xb_bytes(const Dims &d, int64_t q) { return (size_t)(2 * d.o + 1) * (size_t)xb_row_words(q) * 4; }

// segments of the launch preparation: of the longest range of examples, or of the clauses
inline int64_t prep_segments(const Dims &d, int64_t qp) { return (std::max<int64_t>(qp, d.C) + PREP_SEG - 1) / PREP_SEG; }

struct WsLayout {
    size_t tally, ostar, xt, xb, lits, nlit, negcls, gate, ngate, fresh, order, seg_cnt, counters, flag, total;
};

WsLayout ws_layout(const Dims &d, int64_t q)
{
    const int64_t qp = (q + 63) & ~(int64_t)63;
    const int64_t Qw = qp / 32;
    WsLayout L;
    size_t off = 0;
    L.tally = off; off += align256((size_t)d.m * qp * 4);
    L.ostar = off; off += align256((size_t)d.C * Qw * 4);
    L.xt = off; off += align256((size_t)d.Wf * qp * 4);
    L.xb = off; off += align256(xb_bytes(d, q));
    L.lits = off; off += align256((size_t)d.C * LIT_MAX * 4);
    L.nlit = off; off += align256((size_t)d.C * 4);
    L.negcls = off; off += align256((size_t)qp * 4);
    L.gate = off; off += align256((size_t)d.m * qp * 4);
    L.ngate = off; off += align256((size_t)d.m * 4);
    L.fresh = off; off += align256((size_t)d.C * 16);
    L.order = off; off += align256((size_t)d.C * 4);
    L.seg_cnt = off; off += align256((size_t)(d.m + 1) * prep_segments(d, qp) * 8);
    L.counters = off; off += align256((size_t)COUNTER_SETS * 8 * 8);
    L.flag = off; off += 256;
    L.total = off;
    return L;
}

inline int hip_fail(tm_handle *h, hipError_t e)
{
    if (h) h->last_hip = (int)e;
    return TM_EHIP;
}

#define TM_HIP(h, expr)                                  \
    do {                                                 \
        hipError_t e_ = (expr);                          \
        if (e_ != hipSuccess) return hip_fail((h), e_);  \
    } while (0)

inline unsigned blocks_for(int64_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

enum { TIMED_TRAIN = 0, TIMED_PRECALC = 1, TIMED_INFER = 2, TIMED_KINDS = 3 };

// Records an event on the stream when kernel timing is on: called before (first = true)
// and after the launch of a timed kernel.
int timing_mark(tm_handle *h, int kind, bool first, hipStream_t st)
{
    if (!h->timing) return TM_OK;
    if (h->ev_used == h->ev_pool.size()) {
        hipEvent_t e;
        TM_HIP(h, hipEventCreate(&e));
        h->ev_pool.push_back(e);
    }
    TM_HIP(h, hipEventRecord(h->ev_pool[h->ev_used++], st));
    if (first) h->ev_kind.push_back(kind);
    return TM_OK;
}


int fill(tm_handle *h, void *p, size_t bytes, uint32_t v, hipStream_t st)
{
    const int64_t nw = (int64_t)(bytes / 4);
    if (nw == 0) return TM_OK;
    const unsigned nb = (unsigned)std::min<int64_t>(4096, (nw + 255) / 256);
    hipLaunchKernelGGL(k_fill_u32, dim3(nb), dim3(256), 0, st, (uint32_t *)p, nw, v);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

struct EvalPtrs {
    const uint32_t *inc, *X;
    uint32_t *bits;
    int32_t *acc;
};

template <int CH>
void launch_eval_resident(const EvalPtrs &p, const EvalArgs &a, dim3 grid, hipStream_t st)
{
    if (p.bits && p.acc)
        hipLaunchKernelGGL((k_eval_resident<CH, true, true>), grid, dim3(64), 0, st, p.inc, p.X, p.bits, p.acc, a);
    else if (p.bits)
        hipLaunchKernelGGL((k_eval_resident<CH, true, false>), grid, dim3(64), 0, st, p.inc, p.X, p.bits, p.acc, a);
    else
        hipLaunchKernelGGL((k_eval_resident<CH, false, true>), grid, dim3(64), 0, st, p.inc, p.X, p.bits, p.acc, a);
}

// Evaluation of all clauses on q examples; writes bits and/or accumulates sums.
int launch_eval(tm_handle *h, const uint32_t *X, int64_t q, uint32_t *bits, int64_t bits_stride, int32_t *acc,
                int64_t acc_si, int64_t acc_sc, hipStream_t st)
{
    if (q == 0 || (!bits && !acc)) return TM_OK;
    const Dims &d = h->d;
    EvalArgs a;
    const EvalPtrs p{h->inc, X, bits, acc};
    a.q = q; a.Wf = d.Wf; a.W = d.W; a.C = d.C; a.n = d.n; a.m = d.m;
    a.bits_stride = bits_stride; a.acc_si = acc_si; a.acc_sc = acc_sc;
    // a wavefront takes one tile of 64 clauses and a range of examples (a multiple of 256);
    // ranges are sized so that the launch has a few thousand wavefronts per XCD
    const int64_t tiles = (d.C + 63) / 64;
    const int64_t max_ranges = (q + 255) / 256;
    int64_t ranges = (16384 + tiles - 1) / tiles;
    if (ranges > max_ranges) ranges = max_ranges;
    if (ranges > 65535) ranges = 65535;
    if (ranges < 1) ranges = 1;
    int64_t epw = (q + ranges - 1) / ranges;
    epw = (epw + 255) & ~(int64_t)255;
    ranges = (q + epw - 1) / epw;
    a.ex_per_wave = epw;
    const dim3 grid((unsigned)tiles, (unsigned)ranges);
    const int Wf = d.Wf;
    if (Wf <= 1) launch_eval_resident<1>(p, a, grid, st);
    else if (Wf <= 2) launch_eval_resident<2>(p, a, grid, st);
    else if (Wf <= 4) launch_eval_resident<4>(p, a, grid, st);
    else if (Wf <= 8) launch_eval_resident<8>(p, a, grid, st);
    else if (Wf <= 12) launch_eval_resident<12>(p, a, grid, st);
    else if (Wf <= 16) launch_eval_resident<16>(p, a, grid, st);
    else if (Wf <= 20) launch_eval_resident<20>(p, a, grid, st);
    else if (Wf <= 25) launch_eval_resident<25>(p, a, grid, st);
    else if (Wf <= 28) launch_eval_resident<28>(p, a, grid, st);
    else if (Wf <= 32) launch_eval_resident<32>(p, a, grid, st);
    else hipLaunchKernelGGL(k_eval_stream, grid, dim3(64), 0, st, p.inc, p.X, p.bits, p.acc, a);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

struct TrainPtrs {
    const uint32_t *X, *XT, *XB;
    const int32_t *gate, *ngate;
};

template <int WPL>
void launch_train_t(const TrainPtrs &p, const TrainArgs &a, bool full, hipStream_t st)
{
    const size_t lds = (size_t)a.lds_wave_words * TRAIN_WAVES * 4;
    const dim3 grid((unsigned)((a.d.C + TRAIN_WAVES - 1) / TRAIN_WAVES)), block(64 * TRAIN_WAVES);
    if (full) hipLaunchKernelGGL((k_train<WPL, true>), grid, block, lds, st, p.X, p.XT, p.XB, p.gate, p.ngate, a);
    else hipLaunchKernelGGL((k_train<WPL, false>), grid, block, lds, st, p.X, p.XT, p.XB, p.gate, p.ngate, a);
}

// XB (rows of bits over the examples, and the all-ones row) of q examples given row-major.
int build_xb(tm_handle *h, const uint32_t *X, int64_t q, uint32_t *XB, hipStream_t st)
{
    const Dims &d = h->d;
    const int64_t QW = xb_row_words(q);
    hipLaunchKernelGGL(k_transpose_bits, dim3((unsigned)(QW / 2)), dim3(256), 0, st, X, XB, q, d.Wf, d.o, (int)QW);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

// Evaluation of all clauses on the q examples behind XB from their literal lists (rebuilt
// here from the current masks); writes bits and/or the class sums.  With clampT > 0 the
// sums are clamped.  acc need not be zeroed by the caller.
int launch_eval_sparse(tm_handle *h, const uint32_t *XB, int64_t q, uint32_t *lits, int32_t *nlit, uint32_t *bits,
                       int64_t bits_stride, int32_t *acc, int64_t acc_si, int64_t acc_sc, int clampT, int32_t *pred,
                       int32_t *fresh, int timed_kind, hipStream_t st)
{
    const Dims &d = h->d;
    const int64_t QW = xb_row_words(q);
    hipLaunchKernelGGL(k_literal_lists, dim3(blocks_for(d.C, 4)), dim3(256), 0, st, h->inc, lits, nlit, d.C, d.Wf, d.W,
                       d.o, (uint32_t)(QW * 4), fresh, (int)h->qp);
    TM_HIP(h, hipGetLastError());
    SparseArgs a;
    a.bits = bits; a.bits_stride = bits_stride; a.acc = acc; a.acc_si = acc_si; a.acc_sc = acc_sc;
    a.q = q; a.QW = (int)QW; a.QWq = (int)((q + 31) / 32); a.n = d.n; a.m = d.m; a.o = d.o; a.Wf = d.Wf; a.W = d.W;
    // enough workgroups to fill the chip (16 wavefronts each), at most 255 clauses per wavefront,
    // at least 16 clauses per workgroup
    const int64_t ranges = QW / 64;
    int64_t S = (512 + d.m * ranges - 1) / (d.m * ranges);
    S = std::max<int64_t>(S, (d.n + 4079) / 4080);
    S = std::min<int64_t>(S, (d.n + 15) / 16);
    int64_t chunk = (((d.n + S - 1) / S) + 15) & ~(int64_t)15;
    S = (d.n + chunk - 1) / chunk;
    a.S = (int)S; a.chunk = (int)chunk; a.T = (S == 1) ? clampT : 0;
    if (acc && S > 1) {
        // partial sums of several workgroups are added up: start from zero
        if (acc_si == 1) {
            const int rc = fill(h, acc, (size_t)d.m * acc_sc * 4, 0u, st);
            if (rc) return rc;
        } else {
            const int rc = fill(h, acc, (size_t)q * d.m * 4, 0u, st);
            if (rc) return rc;
        }
    }
    int rc = timing_mark(h, timed_kind, true, st);
    if (rc) return rc;
    a.ranges = (int)ranges;
    const int64_t per_xcd = ((ranges + 7) / 8) * d.m * S; // workgroups of the XCD with the most ranges
    a.by_xcd = (ranges >= 24 && per_xcd * 8 <= 0x7fffffff) ? 1 : 0; // few ranges would leave XCDs idle
    const dim3 grid = a.by_xcd ? dim3((unsigned)(per_xcd * 8)) : dim3((unsigned)ranges, (unsigned)(d.m * S));
    hipLaunchKernelGGL(k_eval_sparse, grid, dim3(64 * SP_WAVES), 0, st, lits, nlit, h->inc, XB, a);
    TM_HIP(h, hipGetLastError());
    rc = timing_mark(h, timed_kind, false, st);
    if (rc) return rc;
    // what is left: clamp the added-up sums, pick the class
    if (acc && S > 1 && clampT > 0 && pred)
        hipLaunchKernelGGL(k_clamp_argmax, dim3(blocks_for(q, 256)), dim3(256), 0, st, acc, pred, q, d.m, clampT);
    else if (acc && S > 1 && clampT > 0)
        hipLaunchKernelGGL(k_clamp, dim3(blocks_for(q * d.m, 256)), dim3(256), 0, st, acc, q * d.m, clampT);
    else if (pred)
        hipLaunchKernelGGL(k_argmax, dim3(blocks_for(q, 256)), dim3(256), 0, st, acc, pred, q, d.m);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

// Examples per launch of the training kernel.  Wide clauses (more than 4 register slots
// per lane) evaluate every block from the word-major XT, and an epoch is cut into ranges
// whose slice of XT (Wf rows of `chunk` words) is at most 2 MiB, half of one XCD's L2, so
// that it stays resident while all clauses stream over it (measured: 6x the fetch traffic
// with the whole epoch in one launch).  Narrow clauses sweep through literal rows and do
// better with few launches (measured: one launch of 60,000 examples 0.27 ms against 0.37 ms
// for three): 16 MiB.  Each launch re-reads the tallies for its gate lists.
int64_t train_chunk(const Dims &d)
{
    const int wpl = (d.W + 63) / 64;
    int64_t chunk = ((int64_t)((wpl <= 4 ? 16 : 2) << 20) / (4 * (int64_t)d.Wf)) & ~(int64_t)63;
    if (chunk < 512) chunk = 512;
    return chunk;
}

int launch_train(tm_handle *h, const int32_t *vhat, int64_t i_begin, int64_t i_end, hipStream_t st)
{
    const Dims &d = h->d;
    TrainArgs a;
    const TrainPtrs p{h->X, h->XT, h->XB, h->gate, h->ngate};
    a.d = d; a.sat = h->sat; a.planes = h->planes; a.inc = h->inc; a.tally = h->tally;
    a.vhat = vhat; a.ostar = h->ostar; a.fresh = h->fresh; a.order = h->order; a.counters = h->counters;
    a.q = (int32_t)h->q; a.qp = (int32_t)h->qp; a.Qw = (int32_t)h->Qw; a.epoch = h->epoch;
    a.lds_mask_words = (d.W + 3) & ~3;
    a.lds_off_words = (d.Wf + EVAL_PAD + 3) & ~3;
    a.lds_wave_words = a.lds_mask_words + a.lds_off_words + 2 * ((d.Wf + EVAL_PAD + 1) & ~1) + TRAIN_LIT_MAX + 4;
    a.QW = (int)xb_row_words(h->q);
    const bool full = (d.N == 128);
    const int wpl = (d.W + 63) / 64;
    const int64_t chunk = train_chunk(d);
    h->pairs_visited += (uint64_t)d.C * (uint64_t)(i_end - i_begin);
    for (int64_t b = (i_begin / chunk) * chunk; b < i_end; b += chunk) {
        a.i_begin = (int32_t)std::max(b, i_begin);
        a.i_end = (int32_t)std::min(b + chunk, i_end);
        PrepArgs pa;
        pa.y = h->y; pa.negcls = h->negcls; pa.tally = h->tally; pa.vhat = vhat; pa.fresh = h->fresh;
        pa.gate = h->gate; pa.ngate = h->ngate; pa.order = h->order; pa.seg_cnt = h->seg_cnt; pa.counters = h->counters;
        pa.i_begin = a.i_begin; pa.i_end = a.i_end; pa.qp = a.qp; pa.m = d.m; pa.n = d.n; pa.C = d.C; pa.T = d.T;
        pa.segs = (int)prep_segments(d, h->qp);
        const int64_t items = std::max<int64_t>(a.i_end - a.i_begin, d.C);
        const dim3 pgrid((unsigned)((items + PREP_SEG - 1) / PREP_SEG), (unsigned)(d.m + 1));
        hipLaunchKernelGGL(k_launch_prep<false>, pgrid, dim3(1024), 0, st, pa);
        TM_HIP(h, hipGetLastError());
        hipLaunchKernelGGL(k_launch_prep<true>, pgrid, dim3(1024), 0, st, pa);
        TM_HIP(h, hipGetLastError());
        int rc = timing_mark(h, TIMED_TRAIN, true, st);
        if (rc) return rc;
        if (wpl <= 1) launch_train_t<1>(p, a, full, st);
        else if (wpl <= 2) launch_train_t<2>(p, a, full, st);
        else if (wpl <= 3) launch_train_t<3>(p, a, full, st);
        else if (wpl <= 4) launch_train_t<4>(p, a, full, st);
        else if (wpl <= 6) launch_train_t<6>(p, a, full, st);
        else if (wpl <= 8) launch_train_t<8>(p, a, full, st);
        else if (wpl <= 10) launch_train_t<10>(p, a, full, st);
        else if (wpl <= 12) launch_train_t<12>(p, a, full, st);
        else if (wpl <= 16) launch_train_t<16>(p, a, full, st);
        else if (wpl <= 20) launch_train_t<20>(p, a, full, st);
        else return TM_ELIMIT;
        TM_HIP(h, hipGetLastError());
        rc = timing_mark(h, TIMED_TRAIN, false, st);
        if (rc) return rc;
    }
    return TM_OK;
}

int run_negcls(tm_handle *h, hipStream_t st)
{
    hipLaunchKernelGGL(k_negcls, dim3(blocks_for(h->qp, 256)), dim3(256), 0, st, h->d, h->y, h->negcls, h->q,
                       h->qp, h->epoch);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int fresh_set(tm_handle *h, bool all_stale, hipStream_t st)
{
    hipLaunchKernelGGL(k_fresh_set, dim3(blocks_for(h->d.C, 256)), dim3(256), 0, st, h->fresh, h->d.C, (int)h->qp,
                       all_stale ? 1 : 0);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int sync_tallies(tm_handle *h, hipStream_t st)
{
    const int rc = launch_eval_sparse(h, h->XB, h->q, h->lits, h->nlit, h->ostar, h->Qw, h->tally, 1, h->qp, 0, nullptr,
                                      h->fresh /* every stored output is current afterwards */, TIMED_PRECALC, st);
    return rc;
}

} // namespace

extern "C" {

int tm_state_bytes(const tm_config *cfg, size_t *out)
{
    const int rc = check_config(cfg);
    if (rc) return rc;
    if (!out) return TM_EINVAL;
    const Dims d = make_dims(cfg);
    *out = align256((size_t)d.C * d.W * 8 * 4) + align256((size_t)d.C * d.W * 4);
    return TM_OK;
}

int tm_train_ws_bytes(const tm_config *cfg, int64_t q, size_t *out)
{
    const int rc = check_config(cfg);
    if (rc) return rc;
    if (!out || q < 1) return TM_EINVAL;
    *out = ws_layout(make_dims(cfg), q).total;
    return TM_OK;
}

int tm_create(const tm_config *cfg, void *state_buf, void *stream, tm_handle **out)
{
    const int rc = check_config(cfg);
    if (rc) return rc;
    if (!state_buf || !out || ((uintptr_t)state_buf & 255)) return TM_EINVAL;
    tm_handle *h = new (std::nothrow) tm_handle(); // every member zero, the vectors empty
    if (!h) return TM_EINVAL;
    h->cfg = *cfg;
    h->d = make_dims(cfg);
    const uint32_t top = (uint32_t)(127 + h->d.N), bottom = (uint32_t)(128 - h->d.N);
    for (int b = 0; b < 8; ++b) {
        h->sat.kmax[b] = ((top >> b) & 1u) ? 0u : ~0u;
        h->sat.kmin[b] = ((bottom >> b) & 1u) ? 0u : ~0u;
    }
    h->planes = (uint32_t *)state_buf;
    h->inc = (uint32_t *)((char *)state_buf + align256((size_t)h->d.C * h->d.W * 8 * 4));
    hipError_t e = hipSetDevice(cfg->device);
    if (e != hipSuccess) {
        delete h;
        return TM_EHIP;
    }
    const int64_t nt = (int64_t)h->d.C * h->d.W;
    hipLaunchKernelGGL(k_init_state, dim3(blocks_for(nt, 256)), dim3(256), 0, (hipStream_t)stream, h->d, h->planes,
                       h->inc);
    e = hipGetLastError();
    if (e != hipSuccess) {
        delete h;
        return TM_EHIP;
    }
    *out = h;
    return TM_OK;
}

int tm_destroy(tm_handle *h)
{
    if (!h) return TM_EINVAL;
    for (hipEvent_t e : h->ev_pool) (void)hipEventDestroy(e);
    delete h;
    return TM_OK;
}

int tm_bind_train(tm_handle *h, const uint32_t *X, const int32_t *y, int64_t q, void *ws, void *stream)
{
    if (!h || !X || !y || !ws || q < 1 || ((uintptr_t)ws & 255)) return TM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const Dims &d = h->d;
    // the evaluation loop addresses XT rows with 32-bit byte offsets, and gate-list
    // entries pack the example index into 31 bits
    if ((int64_t)d.Wf * ((q + 63) & ~(int64_t)63) * 4 >= ((int64_t)1 << 32)) return TM_ELIMIT;
    if (q > ((int64_t)1 << 30) - 64) return TM_ELIMIT;
    if (xb_bytes(d, q) >= ((size_t)1 << 32)) return TM_ELIMIT; // literal lists hold 32-bit row offsets
    const WsLayout L = ws_layout(d, q);
    char *base = (char *)ws;
    h->bound = false;
    h->X = X; h->y = y; h->q = q;
    h->qp = (q + 63) & ~(int64_t)63;
    h->Qw = h->qp / 32;
    h->tally = (int32_t *)(base + L.tally);
    h->ostar = (uint32_t *)(base + L.ostar);
    h->XT = (uint32_t *)(base + L.xt);
    h->negcls = (int32_t *)(base + L.negcls);
    h->XB = (uint32_t *)(base + L.xb);
    h->lits = (uint32_t *)(base + L.lits);
    h->nlit = (int32_t *)(base + L.nlit);
    h->gate = (int32_t *)(base + L.gate);
    h->ngate = (int32_t *)(base + L.ngate);
    h->fresh = (int32_t *)(base + L.fresh);
    h->order = (int32_t *)(base + L.order);
    h->seg_cnt = (int32_t *)(base + L.seg_cnt);
    h->counters = (unsigned long long *)(base + L.counters);
    h->flag = (int32_t *)(base + L.flag);

    int rc = fill(h, h->flag, 256, 0u, st);
    if (rc) return rc;
    rc = fill(h, h->counters, (size_t)COUNTER_SETS * 64, 0u, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_check_labels, dim3(blocks_for(q, 256)), dim3(256), 0, st, y, q, d.m, h->flag);
    TM_HIP(h, hipGetLastError());
    int32_t bad = 0;
    TM_HIP(h, hipMemcpyAsync(&bad, h->flag, sizeof(bad), hipMemcpyDeviceToHost, st));
    TM_HIP(h, hipStreamSynchronize(st));
    if (bad) return TM_EINVAL;

    rc = fill(h, h->ostar, (size_t)d.C * h->Qw * 4, 0u, st);
    if (rc) return rc;
    rc = fill(h, h->tally, (size_t)d.m * h->qp * 4, 0u, st);
    if (rc) return rc;
    rc = build_xb(h, X, q, h->XB, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_transpose_x, dim3(blocks_for(h->qp * d.Wf, 256)), dim3(256), 0, st, X, h->XT, q, h->qp,
                       d.Wf);
    TM_HIP(h, hipGetLastError());
    h->bound = true;
    rc = run_negcls(h, st);
    if (rc) return rc;
    return sync_tallies(h, st);
}

int tm_fit_epoch(tm_handle *h, void *stream)
{
    if (!h) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    if (h->epoch >= (1u << 24)) return TM_ELIMIT;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    int rc = run_negcls(h, st);
    if (rc) return rc;
    rc = launch_train(h, nullptr, 0, h->q, st);
    if (rc) return rc;
    h->epoch += 1;
    return TM_OK;
}

int tm_fit_batch(tm_handle *h, int64_t i0, int64_t cnt, void *stream)
{
    if (!h || i0 < 0 || cnt < 0) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    if (i0 > h->q) return TM_EINVAL;
    if (h->epoch >= (1u << 24)) return TM_ELIMIT;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int64_t i_end = (cnt > h->q - i0) ? h->q : i0 + cnt;
    int rc = run_negcls(h, st);
    if (rc) return rc;
    if (i_end <= i0) return TM_OK;
    return launch_train(h, nullptr, i0, i_end, st);
}

int tm_feedback_step(tm_handle *h, const int32_t *tally_snapshot, int64_t i0, int64_t cnt, void *stream)
{
    if (!h || !tally_snapshot || i0 < 0 || cnt < 0) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    if (i0 > h->q) return TM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int64_t i_end = (cnt > h->q - i0) ? h->q : i0 + cnt;
    int rc = run_negcls(h, st);
    if (rc) return rc;
    if (i_end <= i0) return TM_OK;
    return launch_train(h, tally_snapshot, i0, i_end, st);
}

int tm_class_sums(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, void *stream)
{
    if (!h || q < 0) return TM_EINVAL;
    if (q == 0) return TM_OK;
    if (!X || !sums) return TM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const Dims &d = h->d;
    int rc = fill(h, sums, (size_t)q * d.m * 4, 0u, st);
    if (rc) return rc;
    rc = launch_eval(h, X, q, nullptr, 0, sums, d.m, 1, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_clamp, dim3(blocks_for(q * d.m, 256)), dim3(256), 0, st, sums, q * d.m, d.T);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int tm_predict(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, int32_t *sums_scratch, void *stream)
{
    if (!h || q < 0) return TM_EINVAL;
    if (q == 0) return TM_OK;
    if (!pred || !sums_scratch) return TM_EINVAL;
    const int rc = tm_class_sums(h, X, q, sums_scratch, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(k_argmax, dim3(blocks_for(q, 256)), dim3(256), 0, (hipStream_t)stream, sums_scratch, pred, q,
                       h->d.m);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int tm_infer_ws_bytes(const tm_config *cfg, int64_t q, size_t *out)
{
    const int rc = check_config(cfg);
    if (rc) return rc;
    if (!out || q < 0) return TM_EINVAL;
    const Dims d = make_dims(cfg);
    *out = align256(xb_bytes(d, q)) + align256((size_t)d.C * LIT_MAX * 4) + align256((size_t)d.C * 4);
    return TM_OK;
}

// class sums (and, with pred, the decision) of q examples through literal lists; ws as tm_infer_ws_bytes
static int infer_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, int32_t *pred, void *ws, void *stream)
{
    if (!h || q < 0) return TM_EINVAL;
    if (q == 0) return TM_OK;
    if (!X || !sums || !ws || ((uintptr_t)ws & 255)) return TM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const Dims &d = h->d;
    if (xb_bytes(d, q) >= ((size_t)1 << 32)) return TM_ELIMIT;
    char *base = (char *)ws;
    uint32_t *XB = (uint32_t *)base;
    uint32_t *lits = (uint32_t *)(base + align256(xb_bytes(d, q)));
    int32_t *nlit = (int32_t *)(base + align256(xb_bytes(d, q)) + align256((size_t)d.C * LIT_MAX * 4));
    const int rc = build_xb(h, X, q, XB, st);
    if (rc) return rc;
    return launch_eval_sparse(h, XB, q, lits, nlit, nullptr, 0, sums, d.m, 1, d.T, pred, nullptr, TIMED_INFER, st);
}

int tm_class_sums_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, void *ws, void *stream)
{
    return infer_ws(h, X, q, sums, nullptr, ws, stream);
}

int tm_predict_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, int32_t *sums_scratch, void *ws,
                  void *stream)
{
    if (q > 0 && !pred) return TM_EINVAL;
    return infer_ws(h, X, q, sums_scratch, pred, ws, stream);
}

int tm_get_ta_state(tm_handle *h, uint8_t *out, void *stream)
{
    if (!h || !out) return TM_EINVAL;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int64_t nt = (int64_t)h->d.C * h->d.W;
    hipLaunchKernelGGL(k_get_state, dim3(blocks_for(nt, 256)), dim3(256), 0, (hipStream_t)stream, h->d, h->planes,
                       out);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int tm_set_ta_state(tm_handle *h, const uint8_t *in, void *stream)
{
    if (!h || !in) return TM_EINVAL;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int64_t nt = (int64_t)h->d.C * h->d.W;
    hipLaunchKernelGGL(k_set_state, dim3(blocks_for(nt, 256)), dim3(256), 0, (hipStream_t)stream, h->d, in,
                       h->planes, h->inc);
    TM_HIP(h, hipGetLastError());
    if (h->bound) return fresh_set(h, true, (hipStream_t)stream); // stored outputs no longer match the clauses
    return TM_OK;
}

int tm_clause_outputs(tm_handle *h, const uint32_t *X, int64_t q, uint32_t *bits, void *stream)
{
    if (!h || q < 0) return TM_EINVAL;
    if (q == 0) return TM_OK;
    if (!X || !bits) return TM_EINVAL;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    return launch_eval(h, X, q, bits, (q + 31) / 32, nullptr, 0, 0, (hipStream_t)stream);
}

int tm_sync_tallies(tm_handle *h, void *stream)
{
    if (!h) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    return sync_tallies(h, (hipStream_t)stream);
}

int tm_get_tallies(tm_handle *h, int32_t *out, void *stream)
{
    if (!h || !out) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    hipLaunchKernelGGL(k_tally_out, dim3(blocks_for(h->q * h->d.m, 256)), dim3(256), 0, (hipStream_t)stream,
                       h->tally, out, h->q, h->qp, h->d.m);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int tm_get_prev_outputs(tm_handle *h, uint32_t *bits, void *stream)
{
    if (!h || !bits) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int64_t words = (h->q + 31) / 32;
    hipLaunchKernelGGL(k_copy_rows, dim3(blocks_for((int64_t)h->d.C * words, 256)), dim3(256), 0,
                       (hipStream_t)stream, h->ostar, h->Qw, bits, words, (int64_t)h->d.C, words);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int tm_train_chunk(tm_handle *h, int64_t *examples_per_launch)
{
    if (!h || !examples_per_launch) return TM_EINVAL;
    *examples_per_launch = train_chunk(h->d);
    return TM_OK;
}

int tm_set_epoch(tm_handle *h, uint32_t epoch)
{
    if (!h || epoch >= (1u << 24)) return TM_EINVAL;
    h->epoch = epoch;
    return TM_OK;
}

int tm_get_epoch(tm_handle *h, uint32_t *epoch)
{
    if (!h || !epoch) return TM_EINVAL;
    *epoch = h->epoch;
    return TM_OK;
}

int tm_kernel_timing(tm_handle *h, int enable)
{
    if (!h) return TM_EINVAL;
    h->timing = enable != 0;
    h->ev_used = 0;
    h->ev_kind.clear();
    return TM_OK;
}

int tm_read_kernel_timing(tm_handle *h, double *ms, int64_t *launches)
{
    if (!h || !ms || !launches) return TM_EINVAL;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    for (int k = 0; k < TIMED_KINDS; ++k) {
        ms[k] = 0.0;
        launches[k] = 0;
    }
    for (size_t k = 0; k < h->ev_kind.size(); ++k) {
        if (2 * k + 1 >= h->ev_used) break; // a launch that failed between its two marks
        float t = 0.f;
        TM_HIP(h, hipEventSynchronize(h->ev_pool[2 * k + 1]));
        TM_HIP(h, hipEventElapsedTime(&t, h->ev_pool[2 * k], h->ev_pool[2 * k + 1]));
        ms[h->ev_kind[k]] += (double)t;
        launches[h->ev_kind[k]] += 1;
    }
    h->ev_used = 0;
    h->ev_kind.clear();
    return TM_OK;
}

int tm_read_counters(tm_handle *h, uint64_t *out, void *stream)
{
    if (!h || !out) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    unsigned long long tmp[COUNTER_SETS * 8];
    TM_HIP(h, hipMemcpyAsync(tmp, h->counters, sizeof(tmp), hipMemcpyDeviceToHost, st));
    TM_HIP(h, hipStreamSynchronize(st));
    for (int k = 0; k < 8; ++k) {
        out[k] = 0;
        for (int c = 0; c < COUNTER_SETS; ++c) out[k] += tmp[c * 8 + k];
    }
    out[8] = out[0];           // device slot 0: blocks evaluated through literal lists
    out[0] = h->pairs_visited; // every clause visits every example of a pass; known on the host
    h->pairs_visited = 0;
    return fill(h, h->counters, (size_t)COUNTER_SETS * 64, 0u, st);
}

const char *tm_strerror(int code)
{
    switch (code) {
    case TM_OK: return "ok";
    case TM_EINVAL: return "invalid argument or configuration";
    case TM_ESTATE: return "no training data bound (call tm_bind_train first)";
    case TM_EHIP: return "HIP runtime error (see tm_last_hip_error)";
    case TM_ELIMIT: return "size outside the supported range";
    default: return "unknown error code";
    }
}

int tm_last_hip_error(tm_handle *h) { return h ? h->last_hip : 0; }

} // extern "C"
