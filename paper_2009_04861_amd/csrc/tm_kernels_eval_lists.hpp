// Clause evaluation from literal lists, lane = 32 examples (tally pre-calculation, inference with a workspace).
// Part of the one translation unit tm_kernels.hip (included there, in this order).
#ifndef TM_KERNELS_EVAL_LISTS_HPP_
#define TM_KERNELS_EVAL_LISTS_HPP_

namespace tsetlin {

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
// What bounds the kernel is the cache path: every (clause, literal, word of 32 examples) is four
// bytes through the CU's vector L1, which delivers 64 bytes per clock (measured: 0.7 of that rate
// on trained image-like clauses, with 3 of 10 accesses going on to the L2).  Two words per lane
// (8-byte loads, 512 contiguous bytes per wavefront) ran at half the bytes per clock of 4-byte
// loads, with all 32 loads of a round in flight as well as with the registers re-used early: the
// load width is no way round it.

constexpr int LIT_CAP_MIN = 128, LIT_CAP_MAX = 1024; // bounds of the list capacity (entries per clause)
constexpr int SP_WAVES = 8;    // wavefronts per workgroup of k_eval_sparse
constexpr int SP_PLANES = 8;   // bit planes of a wavefront's vote counter: at most 255 clauses per wavefront

// XB from row-major X: workgroups of 4 wavefronts per 64 examples (blockIdx.x) and share of the
// feature words (blockIdx.y), each wavefront a contiguous share of the workgroup's words; the 64 ballots of bit b of a word are two words
// of row 32 fw + b, their complement two words of row o + 32 fw + b.  Examples from q up
// to 32 QW read as feature 0 (no clause output is taken from them).  Row 2o is set to ones.
// (bx, by) = workgroup of a grid of (QW / 2) x ny
__device__ __forceinline__ void transpose_bits_block(const uint32_t *__restrict__ X, uint32_t *__restrict__ XB,
                                                     int64_t q, int Wf, int o, int QW, int bx, int by, int ny)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i = (int64_t)bx * 64 + lane;
    if (threadIdx.x == 0 && by == 0) // these examples' two words of the all-ones row
        *reinterpret_cast<uint2 *>(XB + (int64_t)2 * o * QW + (int64_t)bx * 2) = make_uint2(~0u, ~0u);
    const int per = (Wf + 4 * ny - 1) / (4 * ny);
    const int share = by * 4 + wave;
    const int f_end = min(Wf, (share + 1) * per);
    for (int fw = share * per; fw < f_end; ++fw) {
        const uint32_t x = (i < q) ? X[i * Wf + fw] : 0u;
        uint64_t r = 0;
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            const uint64_t bal = ballot(((x >> b) & 1u) != 0u);
            r = (lane == b) ? bal : r;
        }
        const int k = fw * 32 + lane;
        if (lane < 32 && k < o) {
            *reinterpret_cast<uint2 *>(XB + (int64_t)k * QW + (int64_t)bx * 2) =
                make_uint2((uint32_t)r, (uint32_t)(r >> 32));
            *reinterpret_cast<uint2 *>(XB + (int64_t)(o + k) * QW + (int64_t)bx * 2) =
                make_uint2(~(uint32_t)r, ~(uint32_t)(r >> 32));
        }
    }
}

__global__ __launch_bounds__(256) void k_transpose_bits(const uint32_t *__restrict__ X, uint32_t *__restrict__ XB,
                                                        int64_t q, int Wf, int o, int QW)
{
    transpose_bits_block(X, XB, q, Wf, o, QW, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y);
}

// Literal lists of the clauses, laid out for the wavefronts that walk them.  k_eval_sparse gives
// wavefront w of the workgroup of (class c, share s) the clauses j = s*chunk + w + 8 t of the class
// and walks them in batches of eight (t = 8 b + u, u = 0..7), four list entries of each per round.
// The lists of a batch are therefore interleaved: for batch B = ((c*S + s)*8 + w)*nbatch + b,
//   lits[(B*(cap/4) + k/4)*32 + u*4 + k%4] = entry k of the clause in slot u,   nlit[B*8 + u] = its length,
// so that a round's 32 entries are 128 contiguous bytes behind one pointer (two scalar loads and one
// pointer increment per round instead of eight of each: the kernel is sensitive to the load of
// the CU's scalar unit).  Entry = byte offset of the literal's row in XB; the first `cap` included
// literals in literal order (cap = list capacity, a multiple of 64), the rest of the cap slots
// filled with the all-ones row so that the clauses of a batch can be walked in step; slots of a
// batch beyond the clauses of the share hold the all-ones row throughout and length 0.
// nlit = number of included literals (may exceed cap; such clauses are finished from their masks).
// One wavefront per slot.
struct ListLayout {
    int S, chunk, nbatch; // shares per class, clauses per share, batches per wavefront = ceil(chunk / 64)
    int cap;              // entries per list
};

__device__ __host__ inline int64_t list_slots(int m, const ListLayout &ll) { return (int64_t)m * ll.S * SP_WAVES * ll.nbatch * 8; }

struct ListArgs {
    const uint32_t *inc;
    uint32_t *lits;
    int32_t *nlit;
    int m, n, Wf, W, o;
    ListLayout ll;
    uint32_t row_bytes; // bytes per row of XB
    int32_t *fresh;     // or null
    int qp;
    uint32_t *zero;     // partial sums to clear on the side
    int64_t zero_words;
};

// block = workgroup index within the nblocks workgroups that build the lists
__device__ __forceinline__ void literal_lists_block(const ListArgs &a, int64_t block, int64_t nblocks)
{
    const uint32_t *__restrict__ inc = a.inc;
    uint32_t *__restrict__ lits = a.lits;
    int32_t *__restrict__ nlit = a.nlit;
    const int m = a.m, n = a.n, Wf = a.Wf, W = a.W, o = a.o, qp = a.qp;
    const ListLayout ll = a.ll;
    const uint32_t row_bytes = a.row_bytes;
    int32_t *fresh = a.fresh;
    // on the side: clear the buffer in which the evaluation kernel will add up partial sums
    for (int64_t t = block * 256 + threadIdx.x; t < a.zero_words; t += nblocks * 256) a.zero[t] = 0u;
    // ahead of a tally pre-calculation: every stored output of every clause will be current
    if (fresh)
        for (int64_t g = block * 256 + threadIdx.x; g < (int64_t)m * n; g += nblocks * 256)
            *reinterpret_cast<int4 *>(fresh + g * 4) = make_int4(0, 0, qp, 0);
    const int lane = threadIdx.x & 63;
    const int64_t slot = block * 4 + (threadIdx.x >> 6);
    if (slot >= list_slots(m, ll)) return;
    const int u = (int)(slot & 7);
    const int64_t B = slot >> 3;
    const int b = (int)(B % ll.nbatch);
    const int w = (int)((B / ll.nbatch) % SP_WAVES);
    const int cs = (int)(B / ((int64_t)ll.nbatch * SP_WAVES));
    const int c = cs / ll.S, sh = cs - c * ll.S;
    const int j = sh * ll.chunk + w + SP_WAVES * (8 * b + u);
    const bool real = j < min(n, (sh + 1) * ll.chunk);
    const int g = c * n + (real ? j : 0);
    uint32_t *L = lits + B * (int64_t)(ll.cap / 4) * 32 + u * 4; // entry k at L[(k / 4) * 32 + k % 4]
    const int cap = ll.cap;
    int base = 0;
    for (int w0 = 0; w0 < W && real; w0 += 64) {
        const int lw = w0 + lane;
        uint32_t mk = lw < W ? inc[(int64_t)g * W + lw] : 0u;
        const int cnt = __builtin_popcount(mk);
        int incl = cnt; // inclusive prefix sum over the lanes
#pragma unroll
        for (int dlt = 1; dlt < 64; dlt <<= 1) {
            const int t = __shfl_up(incl, dlt, 64);
            if (lane >= dlt) incl += t;
        }
        int pos = base + incl - cnt;
        const uint32_t k0 = lw >= Wf ? (uint32_t)o + (uint32_t)(lw - Wf) * 32u : (uint32_t)lw * 32u; // literal of bit 0
        while (mk) {
            const int bit = __builtin_ctz(mk);
            mk &= mk - 1u;
            if (pos < cap) L[(pos >> 2) * 32 + (pos & 3)] = (k0 + (uint32_t)bit) * row_bytes;
            ++pos;
        }
        base += __shfl(incl, 63, 64);
    }
    for (int t = min(base, cap) + lane; t < cap; t += 64) L[(t >> 2) * 32 + (t & 3)] = 2u * (uint32_t)o * row_bytes;
    if (lane == 0) nlit[slot] = base;
}

__global__ __launch_bounds__(256) void k_literal_lists(const ListArgs a)
{
    literal_lists_block(a, (int64_t)blockIdx.x, (int64_t)gridDim.x);
}

// Both preparations of an inference call in one launch (they are independent of each other): the first
// nbx * ny workgroups turn the examples into bit rows, the rest build the literal lists.
__global__ __launch_bounds__(256) void k_rows_and_lists(const uint32_t *__restrict__ X, uint32_t *__restrict__ XB, int64_t q,
                                                        int QW, int nbx, int ny, const ListArgs a)
{
    const int64_t nt = (int64_t)nbx * ny;
    if ((int64_t)blockIdx.x < nt)
        transpose_bits_block(X, XB, q, a.Wf, a.o, QW, (int)(blockIdx.x % nbx), (int)(blockIdx.x / nbx), ny);
    else
        literal_lists_block(a, (int64_t)blockIdx.x - nt, (int64_t)gridDim.x - nt);
}

struct SparseArgs {
    uint32_t *bits;      // [C][bits_stride] clause outputs, or null
    int64_t bits_stride;
    int32_t *acc;        // votes of class c for example i go to acc[i*acc_si + c*acc_sc], or null
    int64_t acc_si, acc_sc;
    int64_t q;
    int QW, QWq;         // words per row of XB; words that hold examples (ceil(q/32))
    int n, m, o, Wf, W;
    int lit_cap;         // entries per literal list
    int ranges, by_xcd;  // ranges of 2048 examples; workgroup -> (range, class, share) mapping
    int S, chunk;        // clauses of a class are split over S workgroups, `chunk` (a multiple of 16) each
    int nbatch;          // batches of eight clauses per wavefront: ceil(chunk / 64) (list layout)
    int T;               // > 0: the sums are clamped to [Tlo, T] (only with S = 1)
    int Tlo;             // -T, or 0 in regression mode
    int all_pos;         // regression mode: every clause votes +1
};

// Output of clause g on the 32 examples of this lane's word, taken from its include masks
// (for the rare clause that has more literals than its list holds and is still satisfied somewhere
// after the listed ones); `valid` masks examples >= q.
__device__ __forceinline__ uint32_t clause_from_masks(const uint32_t *__restrict__ inc, const char *xb_lane, int g,
                                                      uint32_t valid, const SparseArgs &a)
{
    uint32_t accv = valid;
    const uint32_t row_bytes = (uint32_t)a.QW * 4u;
    const uint32_t ones_row = 2u * (uint32_t)a.o * row_bytes;
    for (int lw = 0; lw < a.W; ++lw) {
        uint32_t m = inc[(int64_t)g * a.W + lw];
        const uint32_t k0 = lw >= a.Wf ? (uint32_t)a.o + (uint32_t)(lw - a.Wf) * 32u : (uint32_t)lw * 32u;
        while (m) { // four literals of the word per step: four independent loads (the all-ones row where the word runs out)
            uint32_t off[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                off[t] = m ? (k0 + (uint32_t)__builtin_ctz(m)) * row_bytes : ones_row;
                m &= m - 1u; // stays 0 once it is 0
            }
            const uint32_t x0 = *reinterpret_cast<const uint32_t *>(xb_lane + off[0]);
            const uint32_t x1 = *reinterpret_cast<const uint32_t *>(xb_lane + off[1]);
            const uint32_t x2 = *reinterpret_cast<const uint32_t *>(xb_lane + off[2]);
            const uint32_t x3 = *reinterpret_cast<const uint32_t *>(xb_lane + off[3]);
            accv &= x0 & x1 & x2 & x3;
        }
        if (ballot(accv != 0u) == 0) return 0u;
    }
    return accv;
}

// One workgroup per (range of 2048 examples, class c, share s of S).  It evaluates its share
// of the clauses of class c on the range: wavefront w of the 8 takes the clauses j = j_lo + w + 8 k
// (all of one polarity, because j_lo and 8 are even), lane = word of 32 examples.
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
    int64_t B = ((int64_t)cs * SP_WAVES + wave) * a.nbatch; // first batch of this wavefront in the list layout
    for (int j0 = j_lo + wave; j0 < j_hi; j0 += 8 * SP_WAVES, ++B) {
        // eight clauses are walked in step, four literals each per round: 32 loads in flight
        uint32_t x[8];
        int nl[8], longest = 0;
        const int4 *NL = reinterpret_cast<const int4 *>(nlit + B * 8);
        const int4 n0 = NL[0], n1 = NL[1];
        nl[0] = n0.x; nl[1] = n0.y; nl[2] = n0.z; nl[3] = n0.w; nl[4] = n1.x; nl[5] = n1.y; nl[6] = n1.z; nl[7] = n1.w;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u * SP_WAVES;
            x[u] = j < j_hi ? valid : 0u;
            longest = max(longest, min(nl[u], a.lit_cap));
        }
        const uint4 *E = reinterpret_cast<const uint4 *>(lits + B * (int64_t)(a.lit_cap / 4) * 32); // [round][slot] x 4 entries
        for (int k = 0; k < longest; k += 4, E += 8) {
            uint32_t r[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                // past a list's end: the all-ones row.  Row offset (uniform) + word offset (per lane)
                // are added in the vector unit: one operation instead of a 64-bit scalar add per
                // load.  (Buffer loads that take the row offset as their scalar offset need no add
                // at all, but measured 45 % slower: the list entries then sit in scalar registers
                // until their load is issued, and too few list loads stay in flight.)
                const uint4 e = E[u];
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
                if (nl[u] > a.lit_cap && ballot(x[u] != 0u) != 0) x[u] = clause_from_masks(inc, xb_lane, g, valid, a);
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
    const bool positive = (wave & 1) != 0 || a.all_pos; // odd index within the class: positive polarity
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
        if (a.S == 1) *dst = a.T > 0 ? min(max(v, a.Tlo), a.T) : v;
        else if (v) atomicAdd(dst, v);
    }
}

} // namespace tsetlin

#endif
