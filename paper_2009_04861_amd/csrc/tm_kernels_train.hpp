// The training kernel: Algorithm 1, one wavefront per clause.
// Part of the one translation unit tm_kernels.hip (included there, in this order).
#ifndef TM_KERNELS_TRAIN_HPP_
#define TM_KERNELS_TRAIN_HPP_

namespace tsetlin {

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
    const int32_t *y_regr; // regression mode: targets [q] in 0..T; null for classification
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
    int slot_lo, slot_hi; // positions of `order` this launch covers
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
// with more (untrained ones) are swept block by block with eval64.  Trained clauses of the
// image-like workload have 17 literals on average, but a few dozen of 20,000 grow past 64 within
// 30 epochs and past 128 within 100 (always-true negated literals of pixels that are never set
// cost nothing to include); block by block such a clause took 0.45 ms alone when it changed.
constexpr int TRAIN_LIT_MAX = 256;
constexpr int SWEEP_WORDS = 2; // words of 32 examples per lane and pass of a sweep through the literal list

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
// offsets of their rows in XB, padded to a multiple of 8 with the all-ones row; returns
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
    if (lane < 8) llist[min(base, TRAIN_LIT_MAX) + lane] = 2u * (uint32_t)o * xb_row_bytes;
    wave_lds_sync();
    return base;
}

constexpr int TRAIN_WAVES_MAX = 4; // most clauses (wavefronts) per workgroup of the training kernel; the launch chooses

// One wavefront = one clause of class c.  The examples whose gate can open for this
// clause are those of the gate list of c for this launch (label c: trained towards 1;
// drawn negative class c: trained towards 0); their gates are drawn 64 at a time, lane =
// list entry.  Blocks of 64 consecutive examples are evaluated (lane = example) only
// when a gate in them fired or their stored outputs may be outdated; all other blocks
// of the pass are never touched.
// LAZY: the automata (all planes but the include masks) are fetched only when the first feedback
// is due and written back only if there was one; otherwise they are loaded up front.  The kernel
// holds both versions of the loop and picks per clause (see k_train).
template <int WPL, bool FULL, bool REGR, bool LAZY, bool NARROW>
__device__ __forceinline__ void train_clause(const uint32_t *__restrict__ X, const uint32_t *__restrict__ XT,
                                             const uint32_t *__restrict__ XB, const int32_t *__restrict__ gate,
                                             const int k_hi, const TrainArgs &a, uint32_t *lds, const int g,
                                             const int lane, const int wave)
{
    const Dims &d = a.d;
    uint32_t *lmask = lds + wave * a.lds_wave_words;        // [W] include masks, literal-word order
    uint32_t *eoff = lmask + a.lds_mask_words;              // [Wf + EVAL_PAD] (rounded to 4 words)
    uint2 *emask = reinterpret_cast<uint2 *>(eoff + a.lds_off_words);
    uint32_t *llist = lmask + a.lds_wave_words - (TRAIN_LIT_MAX + 8); // [TRAIN_LIT_MAX + 8] literal list for the sweeps

    const int c = g / d.n;
    constexpr bool regr = REGR;                   // regression mode: every clause votes +1 (a compile-time
                                                  // switch: as a run-time one it cost wide clauses 36 registers)
    const bool pos = ((g - c * d.n) & 1) != 0 || regr; // odd index within the class: positive polarity
    const int sign = pos ? 1 : -1;
    const int T = d.T;
    const uint32_t row_bytes = (uint32_t)a.qp * 4u;
    const int i_begin = a.i_begin, i_end = a.i_end, q = a.q;

    // The automata of the clause.  Until the first gate fires only the include masks (plane 7, of
    // which `inc` holds a compact copy) are needed - for evaluation and sweeps -, so the other seven
    // planes are fetched when the first feedback is due and written back only if there was one: in a
    // trained machine most clauses get no feedback in an epoch and move 200 bytes instead of 3.2 KB.
    u32x8 p[WPL];
#pragma unroll
    for (int r = 0; r < WPL; ++r) {
        const int lw = r * 64 + lane;
        u32x8 t = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        if (lw < d.W) t[7] = a.inc[(int64_t)g * d.W + lw];
        p[r] = t;
    }
    bool have_planes = false;
    auto load_planes = [&]() {
#pragma unroll
        for (int r = 0; r < WPL; ++r) {
            const int lw = r * 64 + lane;
            if (lw < d.W) {
                const uint4 *src = reinterpret_cast<const uint4 *>(a.planes + ((int64_t)g * d.W + lw) * 8);
                const uint4 v0 = src[0], v1 = src[1];
                u32x8 t;
                t[0] = v0.x; t[1] = v0.y; t[2] = v0.z; t[3] = v0.w;
                t[4] = v1.x; t[5] = v1.y; t[6] = v1.z; t[7] = v1.w; // equals the include mask held so far
                p[r] = t;
            }
        }
        have_planes = true;
    };
    if (!LAZY) load_planes();
    int nent = build_entries<WPL>(p, lmask, eoff, emask, lane, d.Wf, d.W, row_bytes);

    // lowest Philox block of the Type I comparator that can matter: bits of the
    // uniform below the lowest set bit of thr never decide u < thr
    const int tz = d.thr ? __builtin_ctz(d.thr) : 16;
    const int first_blk = min(tz >> 2, 4);
    const uint32_t ge_init = d.thr >= 65536u ? 0u : ~0u;
    // NARROW (chosen by the host for clauses of at most 16 literal words whose comparison needs more
    // than one Philox block): such clauses leave three quarters of the lanes idle while the 16 word lanes
    // draw up to four blocks each, one after the other, and an epoch of so small a machine costs the
    // latency of its feedback events and nothing else.  Here lane 16 t + w draws block t of word w (one
    // Philox call for all of them) and the word lanes collect the four partial comparisons.  A version of
    // its own because the extra registers would cost the general one-slot kernel a wavefront per SIMD.
    const uint32_t thr_nibble_n = NARROW ? ~(d.thr >> (4 * (lane >> 4))) : 0u; // complement of the four thr bits of this lane's block

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
    const int k_lo = 0;
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
    // of XB, lane = SWEEP_WORDS words of 32 examples: 4096 examples per pass and one load per literal and word.
    int n_listed = -1;          // literals of the current masks (list built if <= TRAIN_LIT_MAX), -1: not counted since the last change
    uint32_t n_changes_v = 0;   // tally changes found by the passes, per lane
    const char *xb_base = reinterpret_cast<const char *>(XB);
    uint32_t *ostar_row = a.ostar + (int64_t)g * a.Qw;
    auto sweep_listed = [&](int bs, int be) { // blocks [bs, be), all of them possibly outdated
        // SWEEP_WORDS words per lane and pass, eight literals per round: 16 independent loads in flight.
        // What a sweep costs is the number of dependent trips to the L2 - a clause whose mask changed
        // walks the rest of the epoch alone, and the last such clause is the tail of the launch
        // (measured per wavefront: 2.6 us per pass of 2,048 examples and 28 literals before, one word
        // per lane).  Four words per lane halve the trips again but cost 24 registers and with them a
        // wavefront per SIMD: 6-8 % on feedback-bound epochs, so two it is.
        const int w_end = 2 * be;
        for (int w0 = 2 * bs; w0 < w_end; w0 += 64 * SWEEP_WORDS) {
            uint32_t rm[SWEEP_WORDS], woff[SWEEP_WORDS], ost[SWEEP_WORDS], accv[SWEEP_WORDS];
#pragma unroll
            for (int u = 0; u < SWEEP_WORDS; ++u) {
                const int w = w0 + u * 64 + lane;
                const bool act = w < w_end;
                const int e0 = w << 5;
                const int lo = min(max(i_begin - e0, 0), 32), hi = min(max(i_end - e0, 0), 32);
                rm[u] = 0u; // examples of the word that belong to this launch
                if (act && hi > lo) rm[u] = (hi == 32 ? ~0u : (1u << hi) - 1u) & ~((1u << lo) - 1u);
                woff[u] = act ? (uint32_t)w * 4u : 0u;
                ost[u] = act ? ostar_row[w] : 0u;
                accv[u] = rm[u];
            }
            for (int k = 0; k < n_listed; k += 8) { // the list is padded to a multiple of 8 with the all-ones row
                const uint4 e = *reinterpret_cast<const uint4 *>(llist + k), e2 = *reinterpret_cast<const uint4 *>(llist + k + 4);
                uint32_t x[SWEEP_WORDS][8];
#pragma unroll
                for (int u = 0; u < SWEEP_WORDS; ++u) {
                    x[u][0] = *reinterpret_cast<const uint32_t *>(xb_base + (e.x + woff[u]));
                    x[u][1] = *reinterpret_cast<const uint32_t *>(xb_base + (e.y + woff[u]));
                    x[u][2] = *reinterpret_cast<const uint32_t *>(xb_base + (e.z + woff[u]));
                    x[u][3] = *reinterpret_cast<const uint32_t *>(xb_base + (e.w + woff[u]));
                    x[u][4] = *reinterpret_cast<const uint32_t *>(xb_base + (e2.x + woff[u]));
                    x[u][5] = *reinterpret_cast<const uint32_t *>(xb_base + (e2.y + woff[u]));
                    x[u][6] = *reinterpret_cast<const uint32_t *>(xb_base + (e2.z + woff[u]));
                    x[u][7] = *reinterpret_cast<const uint32_t *>(xb_base + (e2.w + woff[u]));
                }
                uint32_t any = 0u;
#pragma unroll
                for (int u = 0; u < SWEEP_WORDS; ++u) {
                    accv[u] &= x[u][0] & x[u][1] & x[u][2] & x[u][3] & x[u][4] & x[u][5] & x[u][6] & x[u][7];
                    any |= accv[u];
                }
                // a clause of many literals is false on all examples of the pass after a few rounds
                if (n_listed > 32 && ballot(any != 0u) == 0) break;
            }
#pragma unroll
            for (int u = 0; u < SWEEP_WORDS; ++u) {
                const int w = w0 + u * 64 + lane;
                uint32_t diff = (accv[u] ^ ost[u]) & rm[u];
                if (diff) ostar_row[w] = ost[u] ^ diff;
                n_changes_v += (uint32_t)__builtin_popcount(diff);
                while (diff) { // one tally correction per changed example
                    const int bit = __builtin_ctz(diff);
                    diff &= diff - 1u;
                    atomicAdd(&a.tally[(int64_t)c * a.qp + (w << 5) + bit], ((accv[u] >> bit) & 1u) ? sign : -sign);
                }
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
    auto load_y = [&](int ent) {
        if constexpr (REGR) return ent >= 0 ? a.y_regr[ent >> 1] : 0;
        else return 0;
    };
    // Slot geometry held in registers for the widths whose register budget has room for it (two per slot):
    // which bits of the slot's word are literals at all, and whether they are negated ones.
    constexpr bool GEOM = WPL >= 6 && WPL <= 10;
    uint32_t geom_valid[GEOM ? WPL : 1], geom_neg[GEOM ? WPL : 1];
    if constexpr (GEOM) {
#pragma unroll
        for (int r = 0; r < WPL; ++r) {
            const uint32_t lw = (uint32_t)(r * 64 + lane);
            const bool act = lw < (uint32_t)d.W;
            const bool neg = lw >= (uint32_t)d.Wf;
            const uint32_t fw = neg ? lw - (uint32_t)d.Wf : lw;
            geom_valid[r] = act ? (fw == (uint32_t)d.Wf - 1u ? d.tailmask : ~0u) : 0u;
            geom_neg[r] = neg ? ~0u : 0u;
        }
    }
    int ent_cur = load_ent(k_lo);
    int v_cur = load_v(ent_cur);
    int y_cur = load_y(ent_cur);
    int ent_nxt = load_ent(k_lo + 64);

    for (int k0 = k_lo;; k0 += 64) {
        const bool last = k0 >= k_hi; // all candidates done: one more round sweeps the remaining blocks
        uint64_t fmask = 0, tmask = 0;
        int iv = 0;
        if (!last) {
            const int ent = ent_cur, v = v_cur, yv = y_cur;
            ent_cur = ent_nxt;
            v_cur = load_v(ent_cur);
            y_cur = load_y(ent_cur);
            ent_nxt = load_ent(k0 + 128);
            const bool valid = ent >= 0;
            iv = ent >> 1;
            bool target = (ent & 1) != 0;
            bool fire = false, open = false;
            if (valid) {
                int e, span;
                if (regr) {
                    // regression: error of the clipped vote sum against the target, probability e/T;
                    // below the target the clause is trained towards 1, above it towards 0
                    const int vc = min(max(v, 0), T);
                    target = vc < yv;
                    e = target ? yv - vc : vc - yv;
                    span = T;
                } else {
                    const int vc = min(max(v, -T), T);
                    e = target ? T - vc : T + vc; // Algorithm 1: error of the recorded vote sum
                    span = 2 * T;
                }
                open = e > 0;
                if (open) {
                    const U4 r = draw(d.key, STREAM_GATE, 0, (uint32_t)g, (uint64_t)(uint32_t)iv, a.epoch);
                    fire = (uint64_t)r.x * (uint64_t)span < ((uint64_t)e << 32);
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
            // Type II feedback to a clause whose output is 0 changes nothing (Table 2): no automata needed
            if (LAZY && !have_planes && (tgt == pos || Cout)) load_planes();
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
                        uint32_t lit;
                        if constexpr (GEOM) {
                            valid = geom_valid[r];
                            lit = (xw[r] ^ geom_neg[r]) & valid;
                        } else {
                            lit = literal(lw, xw[r], valid);
                        }
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
                    RngKey key = d.key;
                    uint32_t thr = d.thr;
                    if (WPL <= 2) asm volatile("" : "+s"(key.seed_lo), "+s"(key.seed_hi), "+s"(thr));
                    if constexpr (NARROW) {
                        // Over the four planes of one block the comparison is "the value that went in if
                        // the four bits equal those of thr, else decided": two runs of the chain, from 0
                        // and from 1, give what is decided (d0) and where the input passes (d0 ^ d1).
                        const U4 R = draw(key, STREAM_TYPE1, 4u * (uint32_t)(lane & 15) + (uint32_t)(lane >> 4), (uint32_t)g,
                                          (uint64_t)(uint32_t)ii, a.epoch);
                        const uint32_t w[4] = {R.x, R.y, R.z, R.w};
                        uint32_t d0 = 0u, d1 = ~0u;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const uint32_t K = (uint32_t)__builtin_amdgcn_sbfe((int)thr_nibble_n, k, 1); // thr bit 1: 0, 0: ~0
                            d0 = majority3(w[k], d0, K);
                            d1 = majority3(w[k], d1, K);
                        }
                        const uint32_t pass = d0 ^ d1;
#pragma unroll
                        for (int t = 0; t < 4; ++t) { // least significant block first; lanes 16.. compute nothing that is used
                            const int src = (lane & 15) + 16 * t;
                            const uint32_t dt = (uint32_t)__shfl((int)d0, src, 64), pt = (uint32_t)__shfl((int)pass, src, 64);
                            ge = dt | (pt & ge);
                        }
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            if (t >= first_blk) {
                                // With one or two slots, key and threshold are laundered as well (above):
                                // their derived constants (20 round keys, 16 comparator masks) are then
                                // computed by scalar instructions per slot instead of being kept for the
                                // whole kernel - kept, they overflow the scalar registers and come back
                                // through readlane, a vector instruction each, in the loop that is bound by
                                // vector issue (-5 % per epoch of an untrained machine).  With many slots the
                                // scalar work per slot costs more than the spills (measured +8 .. +20 %).
                                const U4 R = draw(key, STREAM_TYPE1, 4u * lw + (uint32_t)t, (uint32_t)g,
                                                  (uint64_t)(uint32_t)ii, a.epoch);
                                const uint32_t w[4] = {R.x, R.y, R.z, R.w};
#pragma unroll
                                for (int k = 0; k < 4; ++k) {
                                    const uint32_t K = ((thr >> (4 * t + k)) & 1u) ? 0u : ~0u;
                                    ge = majority3(w[k], ge, K);
                                }
                            }
                        }
                    }
                    uint32_t valid;
                    uint32_t lit;
                    if constexpr (GEOM) {
                        valid = geom_valid[r];
                        lit = (xw[r] ^ geom_neg[r]) & valid;
                    } else {
                        lit = literal(lw, xw[r], valid);
                    }
                    uint32_t sp[8];
                    get_slot(p[r], sp);
                    const uint32_t old7 = sp[7];
                    uint32_t up = 0u; // strong: literals that are 1 move towards Include with probability (s-1)/s (1 if boosted)
                    if (Cout) up = lit & (ge | d.boost) & ~at_value<FULL>(sp, a.sat.kmax, true);
                    // weak: everything else moves towards Exclude with probability 1/s
                    const uint32_t wk = (Cout ? ~lit : ~0u) & ~ge & valid & ~at_value<FULL>(sp, a.sat.kmin, false);
                    ripple_updown(sp, up, wk); // the two sets are disjoint: one pass over the planes moves both
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

    if (!LAZY || have_planes) { // a gate fired: the automata may have moved
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
    }
    for (int sh = 32; sh > 0; sh >>= 1) n_changes_v += __shfl_xor(n_changes_v, sh, 64);
    n_changes += n_changes_v;
    // event counters: 64 interleaved sets, because thousands of wavefronts ending at the
    // same time on one address serialise in the L2 atomic unit (measured: ~1.7 ms per launch)
    if (lane < 10) { // slot 4 (trained pairs) is counted by the launch preparation; slot 8: examples this clause
                     // walked; slot 9: 1 if its automata were fetched (and written back)
        const uint32_t v = lane == 0 ? n_listed_blocks : lane == 1 ? n_fired : lane == 2 ? n_type1 : lane == 3 ? n_changes
                         : lane == 4 ? 0u : lane == 5 ? n_type2 : lane == 6 ? n_eval : lane == 7 ? n_draw
                         : lane == 8 ? (uint32_t)(i_end - i_begin) : ((!LAZY || have_planes) ? 1u : 0u);
        if (v) atomicAdd(&a.counters[(g & (COUNTER_SETS - 1)) * COUNTER_WIDTH + lane], (unsigned long long)v);
    }
}

// A clause whose class has many open gates in this launch is all but certain to get feedback: its
// automata are loaded up front and the loop carries no check for them (the check and the pointers it
// keeps alive cost the feedback-bound regime 3-10 %).  With few open gates - a trained machine - most
// clauses get none, and the lazy version saves moving their automata (16 % of a quiet epoch).
constexpr int TRAIN_EAGER_CANDIDATES = 256;

template <int WPL, bool FULL, bool REGR, bool NARROW = false>
__global__ __launch_bounds__(64 * TRAIN_WAVES_MAX) void k_train(const uint32_t *__restrict__ X, const uint32_t *__restrict__ XT,
                                                            const uint32_t *__restrict__ XB,
                                                            const int32_t *__restrict__ gate,
                                                            const int32_t *__restrict__ ngate, const TrainArgs a)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int slot = a.slot_lo + (int)(blockIdx.x * (blockDim.x >> 6)) + wave;
    if (slot >= a.slot_hi) return; // whole wavefront; the kernel has no workgroup-wide barrier
    const int g = __builtin_amdgcn_readfirstlane(a.order[slot]);
    const int k_hi = __builtin_amdgcn_readfirstlane(ngate[g / a.d.n]);
    // wide clauses keep to the one version: the lazy one holds the addresses of all their register slots
    // alive through the loop (36 more registers with 10 slots: one wavefront per SIMD instead of two)
    if (WPL > 4 || k_hi >= TRAIN_EAGER_CANDIDATES) train_clause<WPL, FULL, REGR, false, NARROW>(X, XT, XB, gate, k_hi, a, lds, g, lane, wave);
    else train_clause<WPL, FULL, REGR, WPL <= 4, NARROW>(X, XT, XB, gate, k_hi, a, lds, g, lane, wave);
}

} // namespace tsetlin

#endif
