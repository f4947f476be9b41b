// Preparation of a launch of the training kernel: gate lists per class, launch order of the clauses.
// Part of the one translation unit tm_kernels.hip (included there, in this order).
#ifndef TM_KERNELS_PREP_HPP_
#define TM_KERNELS_PREP_HPP_

namespace tsetlin {

// What a launch of the training kernel over the examples [i_begin, i_end) needs: two stable
// compactions.
//
// Task c < m: gate list of class c = the examples of the range, ascending, whose gate can
// open for a clause of c, packed as (example << 1 | target): target 1 where y_i = c,
// target 0 where c is the class drawn against y_i (regression mode: every example, the bit
// says whether the vote sum lies below the target), and error e > 0 under the tally as it
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
    const int32_t *y, *tally, *vhat, *fresh;
    int32_t *gate, *ngate, *order, *seg_cnt; // seg_cnt [m + 1][segs][2]
    unsigned long long *counters;
    int i_begin, i_end, qp, m, n, C, T, segs;
    int regr; // regression mode: no classes, targets y in [0, T]
    RngKey key;     // the class trained towards 0 for an example is drawn here: uniform over the m - 1 classes other
    uint32_t epoch; // than y_i, a function of (seed, epoch, i) only, so that all clauses agree without communicating
    int g_lo, g_hi; // clauses of the launch (a launch may cover a range of the clauses only)
};

constexpr int COUNTER_SETS = 64; // interleaved copies of the event counters
constexpr int COUNTER_WIDTH = 16; // 64-bit words per copy (9 in use)
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
    const int lo = ordering ? a.g_lo : a.i_begin, hi = ordering ? a.g_hi : a.i_end;
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
            const int yy = a.y[tc], v = vsrc[(int64_t)tc * vstride];
            if (a.regr) { // one bank of clauses: an example is listed unless its clipped vote sum equals its target
                const int vc = min(max(v, 0), a.T);
                tg[r] = live && vc < yy;
                n_seen += live ? 1 : 0;
                f[r] = live && vc != yy;
            } else {
                const U4 u = draw(a.key, STREAM_NEGCLASS, 0, 0, (uint64_t)tc, a.epoch);
                const int dd = (int)(((uint64_t)u.x * (uint64_t)(a.m - 1)) >> 32);
                const int ng = dd + (dd >= yy ? 1 : 0);
                tg[r] = live && yy == c;
                const bool match = live && (tg[r] || ng == c);
                const int vc = min(max(v, -a.T), a.T);
                n_seen += match ? 1 : 0;
                f[r] = match && (tg[r] ? a.T - vc : a.T + vc) > 0; // Algorithm 1: error of the recorded vote sum
            }
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
                atomicAdd(&a.counters[((seg * 16 + wave) & (COUNTER_SETS - 1)) * COUNTER_WIDTH + 4],
                          (unsigned long long)n_seen *
                              (unsigned long long)max(0, min((c + 1) * a.n, a.g_hi) - max(c * a.n, a.g_lo)));
        }
        return;
    }
    __syncthreads();
    int32_t *out = ordering ? a.order + a.g_lo : a.gate + (int64_t)c * a.qp;
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
            out[a.g_hi - a.g_lo - 1 - (before_b + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bb[r] >> 32),
                                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)bb[r], 0u)))] = value;
    }
    // the last segment of a gate list knows its length
    if (!ordering && wave == 0 && lane == 0 && p0 + PREP_SEG >= hi) a.ngate[c] = seg_base[0] + all_f;
}

} // namespace tsetlin

#endif
