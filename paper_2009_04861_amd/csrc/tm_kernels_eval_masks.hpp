// Clause evaluation from include masks, lane = clause (inference without a workspace, clause outputs).
// Part of the one translation unit tm_kernels.hip (included there, in this order).
#ifndef TM_KERNELS_EVAL_MASKS_HPP_
#define TM_KERNELS_EVAL_MASKS_HPP_

namespace tsetlin {

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
    uint64_t posmask;    // lanes of a tile whose clause votes +1: the odd ones, or all in regression mode
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
    const uint64_t cmpos0 = cm0 & a.posmask, cmneg0 = cm0 & ~a.posmask;
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
                    const uint64_t cmpos = cm & a.posmask, cmneg = cm & ~a.posmask;
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
                const uint64_t cmpos = cm & a.posmask; // odd index within class: positive polarity
                const uint64_t cmneg = cm & ~a.posmask;
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

} // namespace tsetlin

#endif
