// HIP kernels and C boundary of the asynchronous Tsetlin machine (gfx950).
// One translation unit: the kernels live in tm_kernels_*.hpp (included below), the device
// helpers (Philox, bit-sliced automata) in tm_device.hpp, the host half of the boundary here.
//
// Memory layout (all device memory is caller-owned):
//   state buffer   planes uint32 [C][W][8]  bit-sliced TA counters, W = 2*Wf literal words
//                  inc    uint32 [C][W]     include masks (= plane 7), compact copy for evaluation
//   train workspace
//                  tally  int32  [m][qp]    voting tallies, qp = q rounded up to 64
//                  ostar  uint32 [C][Qw]    previous clause outputs, 1 bit per (clause, example), Qw = qp/32
//                  XT     uint32 [Wf][qp]   transposed features (word-major) for lane = example evaluation
//                  XB     uint32 [2o+1][QW] literals as bit rows over the examples (row 2o all ones), QW = 64*ceil(q/2048)
//                  lits   uint32 [slots][cap] literal lists of the clauses (cap = 128..1024), interleaved by batches of eight as
//                                           the evaluation kernel walks them (k_literal_lists), nlit int32 [slots] their lengths
//                  gate   int32  [m][qp]    per class and launch: ascending list of (example << 1 | target) whose gate can open
//                  fresh  int32  [C][4]     per clause: example ranges whose stored outputs may be outdated
//                  order  int32  [C]        launch order of the clauses (outdated ones first)
//                  counters uint64 [64][16] interleaved event counters, flag int32
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
#include <mutex>
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
    int regr;          // 1: regression mode (one bank of clauses that all vote +1, targets 0..T)
    uint32_t tailmask; // valid bits of the last feature word
    RngKey key;
};


} // namespace tsetlin

#include "tm_kernels_util.hpp"
#include "tm_kernels_prep.hpp"
#include "tm_kernels_eval_masks.hpp"
#include "tm_kernels_eval_lists.hpp"
#include "tm_kernels_train.hpp"

// ------------------------------------------------------------------------
// host side: handle, validation, launches
// ------------------------------------------------------------------------

// Scratch of tm_predict_static: device memory of the code object itself, so that the call needs no
// caller workspace and allocates nothing.  Every GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: kernels and copies are given the per-device address kept in static_scratch[].
static __device__ __align__(256) unsigned char scratch[TM_STATIC_SCRATCH_BYTES];

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
    uint32_t *XB;   // [2o+1][QW] literal rows of the bound data
    uint32_t *lits; // literal lists, see k_literal_lists
    int32_t *nlit;  // their lengths
    int32_t *gate;  // [m][qp] gate lists of the current launch
    int32_t *ngate; // [m]
    int32_t *fresh;
    int32_t *order; // [C] launch order of the clauses
    int32_t *seg_cnt; // [m + 1][segments][2] flagged items per segment of the launch preparation
    unsigned long long *counters;
    int32_t *flag;
    uint32_t epoch;
    int clause_groups; // sub-launches of consecutive clause ranges per training launch
    int last_hip;
    // kernel timing (measurement aid): event pairs around the launches of the two main kernels
    int timing_kinds;                 // bit k: launches of kind k are bracketed by events
    std::vector<hipEvent_t> ev_pool;  // events created so far, reused
    size_t ev_used;                   // events of the pool handed out since timing was switched on
    std::vector<int> ev_kind;         // kind of the k-th recorded pair (events 2k, 2k+1)
};

namespace {

constexpr int MAX_DEVICES = 64;
void *static_scratch[MAX_DEVICES]; // address of `scratch` on each device, looked up once per device
std::mutex static_scratch_lock;

// Address of this device's copy of `scratch` (the device must be current); null with the HIP error in *err.
void *static_scratch_of(int device, hipError_t *err)
{
    *err = hipSuccess;
    if (device < 0 || device >= MAX_DEVICES) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(static_scratch_lock);
    if (!static_scratch[device]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        static_scratch[device] = p;
    }
    return static_scratch[device];
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int check_config(const tm_config *cfg)
{
    if (!cfg) return TM_EINVAL;
    if (cfg->regression != 0 && cfg->regression != 1) return TM_EINVAL;
    if (cfg->regression ? cfg->n_classes != 1 : cfg->n_classes < 2) return TM_EINVAL;
    if (cfg->clauses_per_class < 2 || (cfg->clauses_per_class & 1)) return TM_EINVAL;
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
    d.regr = cfg->regression ? 1 : 0;
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

// Entries per literal list: a sixteenth of the literals, within [128, 1024], a multiple of 64.
// Trained clauses include far fewer; what does not fit is finished from the include masks.
inline int lit_cap(const Dims &d)
{
    const int want = ((2 * d.o / 16) + 63) & ~63;
    return std::min(LIT_CAP_MAX, std::max(LIT_CAP_MIN, want));
}

// How k_eval_sparse splits the clauses of a class: over S workgroups (8 wavefronts each, three of
// them per CU) of `chunk` clauses (a multiple of 16).  About 1,024 workgroups in all, but at least 256
// clauses per workgroup (zeroing, converting and adding up a workgroup's sums costs as much as walking
// a few hundred clauses), at least 16 per workgroup.  Measured on 10 x 2,000 clauses: 60,000 examples
// 0.23 -> 0.19 ms against one workgroup of 16 wavefronts per CU, 10,000 examples 0.072 -> 0.054 ms.
// A wavefront walks chunk / SP_WAVES clauses and counts their votes in SP_PLANES bit planes, so a
// chunk holds at most (2^SP_PLANES - 1) * SP_WAVES clauses, rounded DOWN to a multiple of 16.
// Returns false if the bound is violated (cannot happen).
inline bool eval_shares(const Dims &d, int64_t ranges, int64_t *S_out, int64_t *chunk_out)
{
    const int64_t chunk_max = (((int64_t)((1 << SP_PLANES) - 1) * SP_WAVES) / 16) * 16;
    int64_t S = (8192 / SP_WAVES + d.m * ranges - 1) / (d.m * ranges);
    S = std::min<int64_t>(S, std::max<int64_t>(1, d.n / 256));
    S = std::max<int64_t>(S, (d.n + chunk_max - 1) / chunk_max);
    S = std::min<int64_t>(S, (d.n + 15) / 16);
    const int64_t chunk = std::min<int64_t>((((d.n + S - 1) / S) + 15) & ~(int64_t)15, chunk_max);
    S = (d.n + chunk - 1) / chunk;
    *S_out = S;
    *chunk_out = chunk;
    return chunk / SP_WAVES < (1 << SP_PLANES) && S * chunk >= d.n && chunk % 16 == 0;
}

// Layout of the literal lists for q examples (see k_literal_lists): depends on how the classes are split.
inline ListLayout list_layout(const Dims &d, int64_t q)
{
    int64_t S = 1, chunk = 16;
    (void)eval_shares(d, xb_row_words(std::max<int64_t>(q, 1)) / 64, &S, &chunk);
    ListLayout ll;
    ll.S = (int)S; ll.chunk = (int)chunk; ll.nbatch = (int)((chunk + 63) / 64); ll.cap = lit_cap(d);
    return ll;
}
inline size_t lits_bytes(const Dims &d, int64_t q) { const ListLayout ll = list_layout(d, q); return (size_t)list_slots(d.m, ll) * ll.cap * 4; }
inline size_t nlit_bytes(const Dims &d, int64_t q) { return (size_t)list_slots(d.m, list_layout(d, q)) * 4; }

struct WsLayout {
    size_t tally, ostar, xt, xb, lits, nlit, gate, ngate, fresh, order, seg_cnt, counters, flag, total;
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
    L.lits = off; off += align256(lits_bytes(d, q));
    L.nlit = off; off += align256(nlit_bytes(d, q));
    L.gate = off; off += align256((size_t)d.m * qp * 4);
    L.ngate = off; off += align256((size_t)d.m * 4);
    L.fresh = off; off += align256((size_t)d.C * 16);
    L.order = off; off += align256((size_t)d.C * 4);
    L.seg_cnt = off; off += align256((size_t)(d.m + 1) * prep_segments(d, qp) * 8);
    L.counters = off; off += align256((size_t)COUNTER_SETS * COUNTER_WIDTH * 8);
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
    if (kind < 0 || !((h->timing_kinds >> kind) & 1)) return TM_OK;
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
    a.posmask = d.regr ? ~0ull : 0xAAAAAAAAAAAAAAAAull;
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

template <int WPL, bool NARROW = false>
void launch_train_t(const TrainPtrs &p, const TrainArgs &a, bool full, hipStream_t st)
{
    // Clauses (wavefronts) per workgroup; the wavefronts of a workgroup do not interact.  Two are best once
    // every SIMD holds several wavefronts (steady epochs of 20,000 clauses: 0.11 ms per launch against
    // 0.14 ms with four; a workgroup's slots are handed on only when its slowest clause is done).  With about
    // one clause per SIMD four are better: they land on the four SIMDs of a CU, while two workgroups of two
    // may share a pair of SIMDs (1,000 clauses: 4.0 ms per epoch against 5.0 ms).
    const int tw = a.d.C <= 1536 ? TRAIN_WAVES_MAX : 2;
    const size_t lds = (size_t)a.lds_wave_words * tw * 4;
    const dim3 grid((unsigned)((a.slot_hi - a.slot_lo + tw - 1) / tw)), block(64 * tw);
    const bool regr = a.y_regr != nullptr;
    if (full && !regr) hipLaunchKernelGGL((k_train<WPL, true, false, NARROW>), grid, block, lds, st, p.X, p.XT, p.XB, p.gate, p.ngate, a);
    else if (!regr) hipLaunchKernelGGL((k_train<WPL, false, false, NARROW>), grid, block, lds, st, p.X, p.XT, p.XB, p.gate, p.ngate, a);
    else if (full) hipLaunchKernelGGL((k_train<WPL, true, true, NARROW>), grid, block, lds, st, p.X, p.XT, p.XB, p.gate, p.ngate, a);
    else hipLaunchKernelGGL((k_train<WPL, false, true, NARROW>), grid, block, lds, st, p.X, p.XT, p.XB, p.gate, p.ngate, a);
}

// XB (rows of bits over the examples, and the all-ones row) of q examples given row-major.
// Grid of the bit transposition: QW / 2 workgroups along the examples, and enough along the feature words
// for a few thousand wavefronts when the examples are few.
inline void xb_grid(const Dims &d, int64_t q, int64_t *nbx, int64_t *ny)
{
    *nbx = xb_row_words(q) / 2;
    *ny = std::max<int64_t>(1, std::min<int64_t>((d.Wf + 3) / 4, (2048 + *nbx - 1) / *nbx));
}

int build_xb(tm_handle *h, const uint32_t *X, int64_t q, uint32_t *XB, hipStream_t st)
{
    const Dims &d = h->d;
    const int64_t QW = xb_row_words(q);
    int64_t wgs_x, split;
    xb_grid(d, q, &wgs_x, &split);
    hipLaunchKernelGGL(k_transpose_bits, dim3((unsigned)wgs_x, (unsigned)split), dim3(256), 0, st, X, XB, q, d.Wf, d.o,
                       (int)QW);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

// Evaluation of all clauses on the q examples behind XB from their literal lists (rebuilt
// here from the current masks); writes bits and/or the class sums.  With clampT > 0 the
// sums are clamped.  acc need not be zeroed by the caller.
int launch_eval_sparse(tm_handle *h, const uint32_t *XB, int64_t q, uint32_t *lits, int32_t *nlit, uint32_t *bits,
                       int64_t bits_stride, int32_t *acc, int64_t acc_si, int64_t acc_sc, int clampT, int32_t *pred,
                       int32_t *fresh, int timed_kind, hipStream_t st, const uint32_t *X_rows = nullptr)
{
    const Dims &d = h->d;
    const int64_t QW = xb_row_words(q);
    SparseArgs a;
    a.bits = bits; a.bits_stride = bits_stride; a.acc = acc; a.acc_si = acc_si; a.acc_sc = acc_sc;
    a.q = q; a.QW = (int)QW; a.QWq = (int)((q + 31) / 32); a.n = d.n; a.m = d.m; a.o = d.o; a.Wf = d.Wf; a.W = d.W; a.lit_cap = lit_cap(d);
    int64_t S, chunk;
    const int64_t ranges = QW / 64;
    if (!eval_shares(d, ranges, &S, &chunk)) return TM_ELIMIT; // cannot happen; guards the vote counters
    const ListLayout ll = list_layout(d, q);
    a.S = (int)S; a.chunk = (int)chunk; a.nbatch = ll.nbatch; a.T = (S == 1) ? clampT : 0;
    a.Tlo = d.regr ? 0 : -a.T; a.all_pos = d.regr;
    // partial sums of several workgroups are added up: they start from zero (either layout, [m][qp] or
    // [q][m]: up to the last element written), cleared by the kernel that builds the lists
    const int64_t zero_words = (acc && S > 1) ? (q - 1) * acc_si + (d.m - 1) * acc_sc + 1 : 0;
    ListArgs la;
    la.inc = h->inc; la.lits = lits; la.nlit = nlit; la.m = d.m; la.n = d.n; la.Wf = d.Wf; la.W = d.W; la.o = d.o;
    la.ll = ll; la.row_bytes = (uint32_t)(QW * 4); la.fresh = fresh; la.qp = (int)h->qp;
    la.zero = reinterpret_cast<uint32_t *>(acc); la.zero_words = zero_words;
    const unsigned list_blocks = blocks_for(list_slots(d.m, ll), 4);
    if (X_rows) { // XB is still to be built from the row-major examples: same launch
        int64_t nbx, ny;
        xb_grid(d, q, &nbx, &ny);
        hipLaunchKernelGGL(k_rows_and_lists, dim3((unsigned)(nbx * ny) + list_blocks), dim3(256), 0, st, X_rows,
                           const_cast<uint32_t *>(XB), q, (int)QW, (int)nbx, (int)ny, la);
    } else {
        hipLaunchKernelGGL(k_literal_lists, dim3(list_blocks), dim3(256), 0, st, la);
    }
    TM_HIP(h, hipGetLastError());
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
        hipLaunchKernelGGL(k_clamp_argmax, dim3(blocks_for(q, 256)), dim3(256), 0, st, acc, pred, q, d.m,
                           d.regr ? 0 : -clampT, clampT, d.regr);
    else if (acc && S > 1 && clampT > 0)
        hipLaunchKernelGGL(k_clamp, dim3(blocks_for(q * d.m, 256)), dim3(256), 0, st, acc, q * d.m,
                           d.regr ? 0 : -clampT, clampT);
    else if (pred)
        hipLaunchKernelGGL(k_argmax, dim3(blocks_for(q, 256)), dim3(256), 0, st, acc, pred, q, d.m, d.regr);
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
    a.y_regr = d.regr ? h->y : nullptr;
    a.vhat = vhat; a.ostar = h->ostar; a.fresh = h->fresh; a.order = h->order; a.counters = h->counters;
    a.q = (int32_t)h->q; a.qp = (int32_t)h->qp; a.Qw = (int32_t)h->Qw; a.epoch = h->epoch;
    a.lds_mask_words = (d.W + 3) & ~3;
    a.lds_off_words = (d.Wf + EVAL_PAD + 3) & ~3;
    a.lds_wave_words = a.lds_mask_words + a.lds_off_words + 2 * ((d.Wf + EVAL_PAD + 1) & ~1) + TRAIN_LIT_MAX + 8;
    a.QW = (int)xb_row_words(h->q);
    const bool full = (d.N == 128);
    const int wpl = (d.W + 63) / 64;
    const int64_t chunk = train_chunk(d);
    for (int64_t b = (i_begin / chunk) * chunk; b < i_end; b += chunk) {
        a.i_begin = (int32_t)std::max(b, i_begin);
        a.i_end = (int32_t)std::min(b + chunk, i_end);
      for (int grp = 0; grp < h->clause_groups; ++grp) {
        // clause ranges of (nearly) equal size; a later group gates on the tallies as the earlier ones left them
        a.slot_lo = (int)((int64_t)d.C * grp / h->clause_groups);
        a.slot_hi = (int)((int64_t)d.C * (grp + 1) / h->clause_groups);
        if (a.slot_hi <= a.slot_lo) continue;
        PrepArgs pa;
        pa.y = h->y; pa.key = d.key; pa.epoch = h->epoch; pa.tally = h->tally; pa.vhat = vhat; pa.fresh = h->fresh;
        pa.gate = h->gate; pa.ngate = h->ngate; pa.order = h->order; pa.seg_cnt = h->seg_cnt; pa.counters = h->counters;
        pa.i_begin = a.i_begin; pa.i_end = a.i_end; pa.qp = a.qp; pa.m = d.m; pa.n = d.n; pa.C = d.C; pa.T = d.T;
        pa.regr = d.regr; pa.g_lo = a.slot_lo; pa.g_hi = a.slot_hi;
        pa.segs = (int)prep_segments(d, h->qp);
        const int64_t items = std::max<int64_t>(a.i_end - a.i_begin, a.slot_hi - a.slot_lo);
        const dim3 pgrid((unsigned)((items + PREP_SEG - 1) / PREP_SEG), (unsigned)(d.m + 1));
        hipLaunchKernelGGL(k_launch_prep<false>, pgrid, dim3(1024), 0, st, pa);
        TM_HIP(h, hipGetLastError());
        hipLaunchKernelGGL(k_launch_prep<true>, pgrid, dim3(1024), 0, st, pa);
        TM_HIP(h, hipGetLastError());
        int rc = timing_mark(h, TIMED_TRAIN, true, st);
        if (rc) return rc;
        // at most 16 literal words and a Type I comparison that needs several Philox blocks (the lowest set bit
        // of the threshold lies below bit 12): the blocks are drawn side by side in the idle lanes
        const bool narrow = d.W <= 16 && d.thr != 0 && __builtin_ctz(d.thr) < 12;
        if (wpl <= 1 && narrow) launch_train_t<1, true>(p, a, full, st);
        else if (wpl <= 1) launch_train_t<1>(p, a, full, st);
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
    }
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
    h->clause_groups = 1;
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
    if (!static_scratch_of(cfg->device, &e)) { // once per device, with that device current
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
    rc = fill(h, h->counters, (size_t)COUNTER_SETS * COUNTER_WIDTH * 8, 0u, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_check_labels, dim3(blocks_for(q, 256)), dim3(256), 0, st, y, q, d.regr ? d.T + 1 : d.m,
                       h->flag);
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
    return sync_tallies(h, st);
}

int tm_fit_epoch(tm_handle *h, void *stream)
{
    if (!h) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    if (h->epoch >= (1u << 24)) return TM_ELIMIT;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int rc = launch_train(h, nullptr, 0, h->q, st);
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
    if (i_end <= i0) return TM_OK;
    return launch_train(h, nullptr, i0, i_end, st);
}

int tm_feedback_step(tm_handle *h, const int32_t *tally_snapshot, int64_t i0, int64_t cnt, void *stream)
{
    if (!h || !tally_snapshot || i0 < 0 || cnt < 0) return TM_EINVAL;
    if (!h->bound) return TM_ESTATE;
    if (i0 > h->q) return TM_EINVAL;
    if (h->epoch >= (1u << 24)) return TM_ELIMIT;
    hipStream_t st = (hipStream_t)stream;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    const int64_t i_end = (cnt > h->q - i0) ? h->q : i0 + cnt;
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
    hipLaunchKernelGGL(k_clamp, dim3(blocks_for(q * d.m, 256)), dim3(256), 0, st, sums, q * d.m, d.regr ? 0 : -d.T,
                       d.T);
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
                       h->d.m, h->d.regr);
    TM_HIP(h, hipGetLastError());
    return TM_OK;
}

int tm_infer_ws_bytes(const tm_config *cfg, int64_t q, size_t *out)
{
    const int rc = check_config(cfg);
    if (rc) return rc;
    if (!out || q < 0) return TM_EINVAL;
    const Dims d = make_dims(cfg);
    *out = align256(xb_bytes(d, q)) + align256(lits_bytes(d, q)) + align256(nlit_bytes(d, q));
    return TM_OK;
}

// class sums (and, with pred, the decision) of q examples through literal lists; ws as tm_infer_ws_bytes
static int infer_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, int32_t *pred, void *ws, void *stream,
                    int timed_kind)
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
    int32_t *nlit = (int32_t *)(base + align256(xb_bytes(d, q)) + align256(lits_bytes(d, q)));
    // the bit rows of the examples and the literal lists are built by one launch
    return launch_eval_sparse(h, XB, q, lits, nlit, nullptr, 0, sums, d.m, 1, d.T, pred, nullptr, timed_kind, st, X);
}

int tm_class_sums_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, void *ws, void *stream)
{
    return infer_ws(h, X, q, sums, nullptr, ws, stream, TIMED_INFER);
}

int tm_predict_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, int32_t *sums_scratch, void *ws,
                  void *stream)
{
    if (q > 0 && !pred) return TM_EINVAL;
    return infer_ws(h, X, q, sums_scratch, pred, ws, stream, TIMED_INFER);
}

int tm_predict_static(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, void *stream)
{
    if (!h || q < 0) return TM_EINVAL;
    if (q == 0) return TM_OK;
    if (!X || !pred) return TM_EINVAL;
    // scratch = workspace of tm_predict_ws followed by its sums_scratch [q][m]
    size_t ws_bytes = 0;
    const int rc = tm_infer_ws_bytes(&h->cfg, q, &ws_bytes);
    if (rc) return rc;
    const size_t need = align256(ws_bytes) + (size_t)q * h->d.m * 4;
    if (need > (size_t)TM_STATIC_SCRATCH_BYTES) return TM_ELIMIT;
    TM_HIP(h, hipSetDevice(h->cfg.device));
    hipError_t e;
    char *base = (char *)static_scratch_of(h->cfg.device, &e); // looked up in tm_create: no HIP call here
    if (!base) return hip_fail(h, e);
    // every word the kernels read is written first by this call (literal rows, lists, lengths; partial sums
    // are cleared by the list kernel), so what an earlier call left in the array does not matter; the
    // kernels are not timed here because recording a new event would allocate
    return infer_ws(h, X, q, (int32_t *)(base + align256(ws_bytes)), pred, base, stream, -1);
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

int tm_eval_shares(const tm_config *cfg, int64_t q, int32_t *shares, int32_t *clauses_per_share)
{
    const int rc = check_config(cfg);
    if (rc) return rc;
    if (q < 1 || !shares || !clauses_per_share) return TM_EINVAL;
    int64_t S, chunk;
    if (!eval_shares(make_dims(cfg), xb_row_words(q) / 64, &S, &chunk)) return TM_ELIMIT;
    *shares = (int32_t)S;
    *clauses_per_share = (int32_t)chunk;
    return TM_OK;
}

int tm_set_clause_groups(tm_handle *h, int32_t groups)
{
    if (!h || groups < 1 || groups > h->d.C) return TM_EINVAL;
    h->clause_groups = groups;
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

int tm_kernel_timing(tm_handle *h, int kinds)
{
    if (!h) return TM_EINVAL;
    if (kinds < 0 || kinds >= (1 << TIMED_KINDS)) return TM_EINVAL;
    h->timing_kinds = kinds;
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
    unsigned long long tmp[COUNTER_SETS * COUNTER_WIDTH];
    TM_HIP(h, hipMemcpyAsync(tmp, h->counters, sizeof(tmp), hipMemcpyDeviceToHost, st));
    TM_HIP(h, hipStreamSynchronize(st));
    uint64_t sum[10];
    for (int k = 0; k < 10; ++k) {
        sum[k] = 0;
        for (int c = 0; c < COUNTER_SETS; ++c) sum[k] += tmp[c * COUNTER_WIDTH + k];
    }
    for (int k = 1; k < 8; ++k) out[k] = sum[k];
    out[0] = sum[8]; // examples walked, summed over the wavefronts (clauses) that ran
    out[8] = sum[0]; // blocks evaluated through literal lists
    out[9] = sum[9]; // (clause, launch) pairs whose automata were moved
    return fill(h, h->counters, (size_t)COUNTER_SETS * COUNTER_WIDTH * 8, 0u, st);
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
