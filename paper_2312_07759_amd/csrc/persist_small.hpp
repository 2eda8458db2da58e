// Persistent kernels for small codebooks: one launch per solve.  Each workgroup
// keeps its tile of W (and of dL/dWq in the backward) in LDS for the whole solve,
// so after the first read no pass touches HBM for its inputs; the only grid-wide
// traffic per pass is one two-hop exchange of O(k d) numbers.
//
// Exchange (per pass over W):
//   hop 1  every workgroup stores its K (D+1) partial sums into its own line of
//          buf1 as 64-bit words {sequence number, float32 value};
//          the first R workgroups are "reducers": reducer r owns a slice of the
//          codewords, reads that slice of every workgroup's line (consecutive
//          lanes read consecutive words), adds them in a fixed order in float64 and
//          applies the O(k d) update (centre update of Alg. 1, or the averaged
//          step of Sec. 4.2) to its slice;
//   hop 2  reducers store the float32 values the next pass needs (codewords, or
//          h/tau) plus a partial residual into buf2; every workgroup reads those
//          few words and takes the same stop decision.
// Value and stamp travel in one atomic word, so no fence and no counter round
// trip is needed; two buffers alternate by sequence parity.  Waits are bounded:
// after spin_limit polls a workgroup raises Ctrl::abort_flag and leaves; the
// others see the flag and leave too.  The grid must fit the device at once.
//
// Exchange of a full-device team (PArgs::tree; 64 or more workgroups, one problem per launch): the hardware hands
// workgroup b to die b mod 8, and workgroups of one die share that die's L2.  A store that only has to reach the
// L2 (workgroup scope) is seen by a device-scope load from the same die after about a third of a microsecond; a word
// that crosses dies has to go through memory and takes more than twice as long.  So:
//   hop 1  (inside a die)  workgroup b stores its partial sums with workgroup scope; workgroup b mod 8, the die's
//          "leader", adds the up to 32 lines of its die in float64 in a fixed order;
//   hop 2  (across dies)   the 8 leaders store their die's totals with device scope; EVERY workgroup reads those 8
//          lines, adds them in the same fixed order and applies the O(k d) update itself, so that all hold the same
//          new state and take the same stop decision without a third hop.
// Every workgroup checks at the start of the launch that it runs on its leader's die (the die index is a hardware
// register); one that does not stores with device scope instead, which is correct on any placement.
#pragma once
#include "common.hpp"
#include "small_k.hpp"

namespace idkm {

constexpr int PT = 256;      // threads per workgroup of the persistent kernels; also the largest grid
constexpr int XLINE = 128;   // words reserved per workgroup in buf1 (K (D+1) <= 80, padded to a power of two)
constexpr int XBCAST = 128;  // words reserved in buf2
constexpr int DIES = 8;      // accelerator dies of the device (each with its own L2); workgroup b runs on die b mod 8
// smallest team that uses the two-level exchange: every die has its leader from DIES workgroups on, and already there it beats
// the one-level form (k = 4, d = 1, per evaluation: 8 workgroups 2.80 -> 2.33 us, 36 workgroups 3.01 -> 2.57, 59 workgroups 3.29 -> 2.86)
constexpr int TREE_MIN_G = DIES;
// Two-level exchange: passes with up to this many sums per workgroup publish per WAVEFRONT (no LDS stage on the sending
// side, hop 2 inside wavefront 0).  With more sums the leader's loads per thread cost more than the senders save:
// measured with 9 .. 16 sums (one 16-word piece per wavefront) against the workgroup-level form below, forward at
// k = 8, d = 1 7.55 against 7.05 us per evaluation, k = 4, d = 2 5.35 against 4.80, (dF/dC)^T pass at k = 16, d = 1
// 6.26 against 5.86; with 32 sums 5.87 against 5.45.
constexpr int WAVE_WORDS_MAX = 8;
#ifndef IDKM_HOP2_PIPE
#define IDKM_HOP2_PIPE 1
#endif
#ifndef IDKM_HOP2_SLEEP
#define IDKM_HOP2_SLEEP 5
#endif
constexpr int HOP2_PIPE = IDKM_HOP2_PIPE;    // loads in flight while waiting for the dies' totals
constexpr int HOP2_SLEEP = IDKM_HOP2_SLEEP;  // s_sleep argument (units of 64 cycles) between their issue
constexpr int XDENSE = 32;   // the explicit-Jacobian mode is offered while its K D (K D + D + 1) sums fit this many words
// Words between the lines of two workgroups in buf1 for a pass with NACC sums per workgroup: shapes of up to 32 sums
// keep the short lines they were tuned with.
constexpr int xline_of(int nacc) { return nacc <= 32 ? 32 : XLINE; }

// What a persistent launch reports; lives in pinned host memory, written once by the kernel.
struct PResult {
    unsigned int done;  // == launch id when the kernel ran to its end
    int iters, converged, nonfinite, halvings;
    double residual, alpha, vnorm;
    int empty[16], bad[16];  // per reducer, from the evaluation at C*
    int nred;                // forward: reducers that report in fin[] (0: the workgroup that wrote `done` wrote everything)
    unsigned int fin[16];    // forward: == launch id once reducer r has written its slice of the state
    int pad_;
};

struct PArgs {
    unsigned long long* buf1;  // [2][PT][xline_of(NACC)] stamped partial sums, word (workgroup, accumulator)
    unsigned long long* buf2;  // [2][XBCAST] stamped broadcast values
    unsigned long long* buf3;  // [2][DIES][XLINE] two-level exchange: stamped totals of each die
    unsigned long long* tab;   // [DIES] two-level exchange: die index of each leader, stamped with the launch id
    int tree;                  // two-level exchange (team of at least TREE_MIN_G workgroups, one problem per launch);
                               // 2: the same with every store at device scope (test support)
    int gm_basis;              // backward, BWD_GMRES: longest Krylov basis before a restart
    unsigned int gm_off;       // backward, BWD_GMRES: byte offset of the solve's state in the dynamic LDS (a multiple of 16)
    unsigned int seq_base;     // sequence numbers seq_base+1 ... are used by this launch; seq_base+1 is its id
    unsigned int spin_limit;   // polls before a wait gives up
    int per;                   // vectors per workgroup tile
    const float* C0;           // forward: initial codebook [k,d]
    double tol;                // stop rule of the solve (forward: absolute; backward: relative to ||v||)
    int max_iter;
    int mode;                  // backward: BWD_IMPLICIT or BWD_JFB
    double alpha;              // backward: damping factor
    unsigned int* abort_word;  // device word; holds this launch's id once a bounded wait has expired
    PResult* out;              // pinned host memory
    int wg, G;                 // this workgroup's index within its team and the team's size; filled in by the kernel
#ifdef IDKM_TRACE
    long long* trace;          // [2 workgroups][64 passes][8 stamps], then [256 workgroups][8 stamps] of pass 20 (development builds only)
#endif
};

// One problem of a batched launch: the workgroups [wg_begin, wg_begin + wg_count) of the grid form its team.
struct BatchItem {
    Args a;
    PArgs p;
    int wg_begin, wg_count;
};

#ifdef IDKM_TRACE
#define IDKM_STAMP(slot)                                                                                  \
    do {                                                                                                  \
        if (pa.trace && threadIdx.x == 0 && s_iters < 64 && (pa.wg == 0 || pa.wg == pa.G - 1))             \
            pa.trace[((pa.wg == 0 ? 0 : 1) * 64 + s_iters) * 8 + (slot)] = (long long)clock64();           \
        if (pa.trace && threadIdx.x == 0 && s_iters == 20 && pa.wg < 256)                                  \
            pa.trace[2 * 64 * 8 + pa.wg * 8 + (slot)] = (long long)wall_clock64();                              \
    } while (0)
#define IDKM_SUB(slot)                                                                       \
    do {                                                                                     \
        if (pa.trace && threadIdx.x == 0 && pa.wg == 0)                                      \
            pa.trace[2 * 64 * 8 + 256 * 8 + (slot)] = (long long)clock64();                  \
    } while (0)
#else
#define IDKM_STAMP(slot) do { } while (0)
#define IDKM_SUB(slot) do { } while (0)
#endif


// Shared scratch of the exchange.
template <int NACC>
struct XShared {
    float rpart[pow2_at_least(NACC)][PT / 64];  // partial sums of every wavefront, [accumulator][wavefront]
    double red2[PT];                 // reducer: per-thread sums (thread t: word t mod WPR, workgroups t/WPR + k PT/WPR)
    double tot[8];                   // reducer: totals of its slice
    unsigned int bc[XBCAST];         // payloads of the broadcast words
    float own[XLINE];                // this workgroup's own partial sums (read back directly by a team of one)
    int abort;
    // two-level exchange
    int local;                       // this workgroup runs on its leader's die: its partial sums need only reach the L2
    float stage2[DIES * (NACC <= 8 ? 8 : NACC)];  // totals of the dies, [die][slot]
    double totd[NACC];               // grid totals
};

// Between LDS accesses of ONE wavefront where a lane reads what another lane wrote: the hardware runs a wavefront's
// LDS instructions in order, but the compiler reasons per thread (it may forward a thread's own earlier load past
// another lane's store, or move accesses); this keeps its memory operations in program order.  No instruction issued
// beyond a wait for the outstanding LDS operations.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Index of the accelerator die this wavefront runs on.
__device__ __forceinline__ unsigned int die_id() {
    unsigned int v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return v & 0xfu;
}
// A stamped word that only a workgroup of the same die will read: it has to reach the die's L2, not memory.
__device__ __forceinline__ void st_word_die(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
// Sum over the four lanes l % 16 + 16 r of a wavefront (one lane of each row of 16), in every lane.
// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second, v_permlane32_swap
// the upper half of the first with the lower half of the second; adding the two results pairs every lane with its
// partner, and both partners add the same two numbers (in either order: the same sum).
__device__ __forceinline__ float cross_row_sum(float x) {
    u32x2_t s = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(s[0]) + __uint_as_float(s[1]);
    s = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(s[0]) + __uint_as_float(s[1]);
}
__device__ __forceinline__ double cross_row_sum_d(double x) {
    u32x2_t lo = __builtin_amdgcn_permlane16_swap((unsigned)__double2loint(x), (unsigned)__double2loint(x), false, false);
    u32x2_t hi = __builtin_amdgcn_permlane16_swap((unsigned)__double2hiint(x), (unsigned)__double2hiint(x), false, false);
    x = __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
    lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(x), (unsigned)__double2loint(x), false, false);
    hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(x), (unsigned)__double2hiint(x), false, false);
    return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}
// Row totals of accumulators [OFF, NACC) into xs.rpart, taken in power-of-two pieces, largest first (80 sums are a
// piece of 64 and one of 16, not one of 128 padded with zeros: the exchange network costs about three instructions
// per value it starts with).
constexpr int pow2_at_most(int n) {
    int p = 2;
    while (2 * p <= n) p *= 2;
    return p;
}
template <int NACC, int OFF, class XS>
__device__ __forceinline__ void publish_rows(const float (&acc)[NACC], XS& xs, int lane, int wave) {
    constexpr int NP = pow2_at_most(NACC - OFF);
    float v[NP];
#pragma unroll
    for (int q = 0; q < NP; ++q) v[q] = (OFF + q < NACC) ? acc[OFF + q] : 0.f;
    row_sums<NP>(v, lane);
    // the four rows of the wavefront in registers (two row swaps per value), so that LDS only sees one value per
    // wavefront and accumulator
#pragma unroll
    for (int i = 0; i < row_sum_live(NP); ++i) v[i] = cross_row_sum(v[i]);
    if (lane < 16 && row_sum_owner<NP>(lane)) {
#pragma unroll
        for (int i = 0; i < row_sum_live(NP); ++i) {
            const int q = OFF + row_sum_index<NP>(lane, i);
            if (q < NACC) xs.rpart[q][wave] = v[i];
        }
    }
    if constexpr (OFF + NP < NACC) publish_rows<NACC, OFF + NP>(acc, xs, lane, wave);
}

// hop 1, sender side: workgroup partial of every accumulator into this workgroup's line.
template <int NACC, class XS>
__device__ __forceinline__ void publish_waves(const PArgs& pa, unsigned int seq, const float (&acc)[NACC], XS& xs);
template <int NACC, class XS>
__device__ __forceinline__ void publish_partials(const PArgs& pa, unsigned int seq, const float (&acc)[NACC], XS& xs) {
    const int tid = threadIdx.x, lane = tid & 63;
    if constexpr (NACC <= WAVE_WORDS_MAX) {
        if (pa.tree) {
            publish_waves<NACC>(pa, seq, acc, xs);
            return;
        }
    }
    IDKM_SUB(0);
    publish_rows<NACC, 0>(acc, xs, lane, tid >> 6);
    IDKM_SUB(1);
    __syncthreads();
    IDKM_SUB(2);
    if (tid < NACC) {
        // the four wavefronts in float64, a fixed order
        const double s = ((double)xs.rpart[tid][0] + (double)xs.rpart[tid][1]) +
                         ((double)xs.rpart[tid][2] + (double)xs.rpart[tid][3]);
        xs.own[tid] = (float)s;
        // a workgroup's words lie together: one store transaction per workgroup and pass
        unsigned long long* dst = &pa.buf1[((size_t)(seq & 1u) * PT + pa.wg) * xline_of(NACC) + tid];
        if (!pa.tree)
            st_word(dst, pack_f(seq, (float)s));
        else if (pa.wg >= DIES) {  // (a leader reads its own sums from xs.own)
            if (xs.local)
                st_word_die(dst, pack_f(seq, (float)s));
            else
                st_word(dst, pack_f(seq, (float)s));
        }
    }
    IDKM_SUB(3);
}

// Bounded wait for NW stamped words (src, src + stride, ...) of this thread.  Returns false if the wait was
// abandoned.  (Keeping several polls in flight does not shorten the wait: it is the store's way to the other
// dies that takes the time, not the phase of the poll.)
template <int NW>
__device__ __forceinline__ bool poll_words(const PArgs& pa, const unsigned long long* src, size_t stride,
                                           unsigned int seq, unsigned long long (&out)[NW]) {
    unsigned int spins = 0;
    for (;;) {
#pragma unroll
        for (int q = 0; q < NW; ++q) out[q] = ld_word(src + q * stride);
        bool ok = true;
#pragma unroll
        for (int q = 0; q < NW; ++q) ok = ok && ((unsigned int)(out[q] >> 32) == seq);
        if (ok) return true;
        ++spins;
        if (spins > pa.spin_limit ||
            ((spins & 31u) == 0u && __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u))
            return false;
    }
}

// Bounded wait for ONE stamped word with PIPE loads in flight, issued SLEEP x 64 cycles apart: a load that has to go
// to memory returns after more than half a microsecond, so with one load at a time a word that lands just after a load
// was issued is seen a whole round trip later; with staggered loads the next one is at most a fraction of that away.
template <int PIPE, int SLEEP>
__device__ __forceinline__ bool poll_word_staggered(const PArgs& pa, const unsigned long long* src, unsigned int seq,
                                                    unsigned long long& out) {
    unsigned long long w[PIPE];
#pragma unroll
    for (int i = 0; i < PIPE; ++i) {
        w[i] = ld_word(src);
        if (i + 1 < PIPE) __builtin_amdgcn_s_sleep(SLEEP);
    }
    unsigned int spins = 0;
    for (;;) {
#pragma unroll
        for (int i = 0; i < PIPE; ++i) {
            if ((unsigned int)(w[i] >> 32) == seq) {
                out = w[i];
                return true;
            }
            w[i] = ld_word(src);
        }
        spins += PIPE;
        if (spins > pa.spin_limit ||
            ((spins & 31u) < (unsigned)PIPE && __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u))
            return false;
    }
}

// hop 1, reducer side: totals over all workgroups of words [first, first+WPR) into xs.tot (float64, fixed order).
// Returns false if the wait was abandoned (uniform over the workgroup).
template <int NACC, int WPR, class XS>
__device__ __forceinline__ bool reduce_slice(const PArgs& pa, unsigned int seq, int first, XS& xs) {
    static_assert(WPR <= 8, "a reducer handles at most 8 words per workgroup");
    const int tid = threadIdx.x;
    IDKM_SUB(4);
    const int G = pa.G;
    constexpr int GPT = PT / WPR;                 // workgroups one load instruction of the whole workgroup covers
    constexpr int NL = (PT + GPT - 1) / GPT;      // loads per thread that cover PT workgroups
    constexpr int PER = (GPT + 31) / 32;          // per-thread sums one thread of the second stage adds
    // every workgroup's words lie together (one store transaction per workgroup); the reducer reads them as one flat
    // array, thread t taking word t mod WPR of workgroups t/WPR, t/WPR + GPT, ...: consecutive lanes, consecutive words
    const int q = tid % WPR, g0 = tid / WPR;
    double s = 0.0;
    bool aborted = false;
    if (G == 1) {
        // a team of one has nobody to wait for: its partial sums are the totals
        __syncthreads();
        if (tid < WPR) s = (double)xs.own[first + tid];
    } else if (g0 < GPT && g0 < G) {
        constexpr int LINE = xline_of(NACC);
        const unsigned long long* src = pa.buf1 + ((size_t)(seq & 1u) * PT + g0) * LINE + first + q;
        const int nv = (G - g0 + GPT - 1) / GPT;  // <= NL
        unsigned int spins = 0;
        for (;;) {
            unsigned long long w[NL];
#pragma unroll
            for (int u = 0; u < NL; ++u) w[u] = (u < nv) ? ld_word(src + (size_t)u * GPT * LINE) : pack_f(seq, 0.f);
            bool ok = true;
#pragma unroll
            for (int u = 0; u < NL; ++u) ok = ok && ((unsigned int)(w[u] >> 32) == seq);
            if (ok) {
#pragma unroll
                for (int u = 0; u < NL; ++u) s += (double)__uint_as_float((unsigned int)w[u]);
                break;
            }
            ++spins;
            if (spins > pa.spin_limit ||
                ((spins & 31u) == 0u && __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u)) {
                aborted = true;
                break;
            }
        }
    }
    IDKM_SUB(5);
    xs.red2[tid] = s;
    if (aborted) {
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
#ifdef IDKM_TRACE
    if (pa.trace && threadIdx.x == 0 && pa.wg == 0) pa.trace[2 * 64 * 8 - 1] = (long long)clock64();
#endif
    if (xs.abort) return false;
    IDKM_SUB(6);
    // thread (qq, part) adds PER consecutive per-thread sums of word qq, then a fixed 32-lane DPP network
    const int qq = tid >> 5, part = tid & 31;
    double t = 0.0;
    if (qq < WPR) {
#pragma unroll
        for (int v = 0; v < PER; ++v) {
            const int g = part * PER + v;
            if (g < GPT) t += xs.red2[g * WPR + qq];
        }
    }
    t = half_sum_d_dpp(t);
    if (qq < WPR && part == 31) xs.tot[qq] = t;
    __syncthreads();
    IDKM_SUB(7);
    return true;
}

// hop 2, receiver side: waits for words [0, nwords) of buf2 and leaves their payloads in xs.bc.  Words
// [0, KD) belong to slices of WPR words, word KD + r to reducer r; a reducer has put the words of its own slices
// into xs.bc already and does not wait for the round trip of its own stores.
template <int NACC, int WPR, int KD, class XS>
__device__ __forceinline__ bool gather_bcast(const PArgs& pa, unsigned int seq, int nwords, bool keep_own, XS& xs) {
    const int tid = threadIdx.x;
    bool aborted = false;
    const int slice = (tid < KD) ? tid / WPR : tid - KD;
    if (tid < nwords && !(keep_own && (slice % pa.G) == pa.wg)) {
        const unsigned long long* src = pa.buf2 + (size_t)(seq & 1u) * XBCAST + tid;
        unsigned long long w[1];
        if (poll_words<1>(pa, src, 0, seq, w))
            xs.bc[tid] = (unsigned int)w[0];
        else
            aborted = true;
    }
    if (aborted) {
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return xs.abort == 0;
}

// ---------------------------------------------------------------- two-level exchange (PArgs::tree)

// Start of a launch: the leaders publish the die they run on; every workgroup compares it with its own.
// Leaves xs.local; returns false if the wait was abandoned.  Called by all threads; ends with a barrier.
// (the leaders say where they run before they load their tile -- tree_announce -- so that nobody waits for that word)
__device__ __forceinline__ void tree_announce(const PArgs& pa) {
    if (pa.tree && threadIdx.x == 0 && pa.wg < DIES) st_word(&pa.tab[pa.wg], pack_u(pa.seq_base + 1u, die_id()));
}
template <class XS>
__device__ __forceinline__ bool tree_handshake(const PArgs& pa, XS& xs) {
    if (threadIdx.x == 0) {
        const unsigned int id = pa.seq_base + 1u, mine = die_id();
        int local = 1;
        if (pa.wg >= DIES) {
            unsigned long long w[1];
            if (poll_words<1>(pa, pa.tab + (pa.wg % DIES), 0, id, w)) {
                local = ((unsigned int)w[0] == mine) ? 1 : 0;
            } else {
                xs.abort = 1;
                __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (pa.tree == 2) local = 0;  // test support: behave as if no workgroup ran on its leader's die
        xs.local = local;
    }
    __syncthreads();
    return xs.abort == 0;
}

// hop 1, leader side (workgroups 0 .. DIES-1): totals of the partial sums of workgroups wg, wg + DIES, ... in
// float64, published as the die's line of buf3 and left in xs.stage2 for this workgroup's own hop 2.  Thread t takes
// accumulator t % NACC of members t / NACC, t / NACC + PARTS, ... and adds them in registers in increasing order (two
// interleaved chains); the PARTS groups are added through LDS, again in a fixed order.  Returns false if the wait was
// abandoned (uniform over the workgroup).
template <int NACC, class XS>
__device__ __forceinline__ bool tree_die_totals(const PArgs& pa, unsigned int seq, XS& xs) {
    constexpr int LINE = xline_of(NACC);
    constexpr int PARTS = PT / NACC;                 // member groups
    constexpr int MPT = (32 + PARTS - 1) / PARTS;    // members per thread
    static_assert(PARTS >= 1, "one thread per accumulator at least");
    const int tid = threadIdx.x, x = pa.wg, q = tid % NACC, part = tid / NACC;
    const bool live = part < PARTS;
    const int nmem = (pa.G - x + DIES - 1) / DIES;  // members of this die, the leader included; <= 32
    const unsigned long long* line0 = pa.buf1 + ((size_t)(seq & 1u) * PT + x) * LINE + q;
    unsigned long long w[MPT];
    bool valid[MPT];
#pragma unroll
    for (int u = 0; u < MPT; ++u) {
        const int mi = part + PARTS * u;
        valid[u] = live && mi >= 1 && mi < nmem;  // member 0 is this workgroup: its sums are in xs.own
    }
    bool aborted = false;
    unsigned int spins = 0;
    for (;;) {
#pragma unroll
        for (int u = 0; u < MPT; ++u)
            w[u] = valid[u] ? ld_word(line0 + (size_t)(part + PARTS * u) * DIES * LINE) : pack_f(seq, 0.f);
        bool ok = true;
#pragma unroll
        for (int u = 0; u < MPT; ++u) ok = ok && ((unsigned int)(w[u] >> 32) == seq);
        if (ok) break;
        ++spins;
        if (spins > pa.spin_limit ||
            ((spins & 31u) == 0u && __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u)) {
            aborted = true;
            break;
        }
    }
    if (live) {
        // (thread q < NACC wrote xs.own[q] itself in publish_partials; members that do not exist carry zeros)
        double c2[2] = {tid < NACC ? (double)xs.own[q] : 0.0, 0.0};
#pragma unroll
        for (int u = 0; u < MPT; ++u) c2[u & 1] += (double)__uint_as_float((unsigned int)w[u]);
        xs.red2[part * NACC + q] = c2[0] + c2[1];
    }
    if (aborted) {
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (xs.abort) return false;
    if (tid < NACC) {
        double c2[2] = {0.0, 0.0};
#pragma unroll
        for (int g = 0; g < PARTS; ++g) c2[g & 1] += xs.red2[g * NACC + tid];
        const float tot = (float)(c2[0] + c2[1]);
        xs.stage2[x * NACC + tid] = tot;
        st_word(&pa.buf3[((size_t)(seq & 1u) * DIES + x) * LINE + tid], pack_f(seq, tot));
    }
    return true;
}

// hop 2, every workgroup: waits for the totals of the DIES dies and adds them in float64 in a fixed order; the grid
// totals are left in xs.totd.  Ends with a barrier.  Returns false if the wait was abandoned.
template <int NACC, class XS>
__device__ __forceinline__ bool tree_grid_totals(const PArgs& pa, unsigned int seq, XS& xs) {
    constexpr int LINE = xline_of(NACC);
    constexpr int NLD = (DIES * NACC + PT - 1) / PT;
    const int tid = threadIdx.x;
    const unsigned long long* base = pa.buf3 + (size_t)(seq & 1u) * DIES * LINE;
    unsigned long long w[NLD];
    bool valid[NLD];
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
        const int f = tid + u * PT, x = f / NACC;
        valid[u] = f < DIES * NACC && x != pa.wg;  // a leader has left its own die's totals in xs.stage2 already
    }
    bool aborted = false;
    unsigned int spins = 0;
    for (;;) {
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int f = tid + u * PT, x = f / NACC, q = f - x * NACC;
            w[u] = valid[u] ? ld_word(base + (size_t)x * LINE + q) : pack_f(seq, 0.f);
        }
        bool ok = true;
#pragma unroll
        for (int u = 0; u < NLD; ++u) ok = ok && ((unsigned int)(w[u] >> 32) == seq);
        if (ok) break;
        ++spins;
        if (spins > pa.spin_limit ||
            ((spins & 31u) == 0u && __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u)) {
            aborted = true;
            break;
        }
    }
#pragma unroll
    for (int u = 0; u < NLD; ++u)
        if (valid[u]) xs.stage2[tid + u * PT] = __uint_as_float((unsigned int)w[u]);
    if (aborted) {
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (xs.abort) return false;
    if (tid < NACC) {
        double t[DIES];
#pragma unroll
        for (int x = 0; x < DIES; ++x) t[x] = (double)xs.stage2[x * NACC + tid];
        xs.totd[tid] = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
    }
    __syncthreads();
    return true;
}


// ---------------------------------------------------------------- two-level exchange, up to 8 sums per workgroup

// The shapes whose passes leave at most 8 sums per workgroup (k = 2 and k = 4 with scalar weights in the forward loop, k d <= 8
// in the backward passes) take the two-level exchange without a detour through LDS on the sending side: every
// WAVEFRONT reduces its lanes' sums to one value each (the halving network inside rows of 16 lanes, then two row
// swaps) and stores its own 8 words; the leader adds 4 wavefronts x up to 32 workgroups, again across lanes, and hop
// 2 runs inside wavefront 0 of every workgroup.  Slot p of a line holds accumulator slot_acc(p) (the order in which
// the halving network leaves them in the lanes); unused slots carry zeros.
__host__ __device__ constexpr int slot_acc(int p) { return (p & 1) * 4 + ((p >> 1) & 1) * 2 + ((p >> 2) & 1); }
// Sum over the eight lanes that share l % 8 (lanes l, l + 8, ..., l + 56), in every lane, float64, fixed order.
__device__ __forceinline__ double sum_over_lane_bits_3_to_5(double x) {
    x += dpp_d<0x128, 0xf>(x);  // row_ror:8
    return cross_row_sum_d(x);
}

// hop 1, sender side: every wavefront stores the totals of its lanes' sums as 8 stamped words.
template <int NACC, class XS>
__device__ __forceinline__ void publish_waves(const PArgs& pa, unsigned int seq, const float (&acc)[NACC], XS& xs) {
    static_assert(NACC <= 8, "one 8-word piece per wavefront");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = (q < NACC) ? acc[q] : 0.f;
    row_sums<8>(v, lane);  // lane l of a row: the row's total of accumulator slot_acc(l % 8)
    const float tot = cross_row_sum(v[0]);
    if (lane < 8) {
        xs.own[wave * 8 + lane] = tot;
        if (pa.wg >= DIES) {  // (a leader reads its own sums from xs.own)
            unsigned long long* dst = &pa.buf1[((size_t)(seq & 1u) * PT + pa.wg) * 32 + wave * 8 + lane];
            if (xs.local)
                st_word_die(dst, pack_f(seq, tot));
            else
                st_word(dst, pack_f(seq, tot));
        }
    }
}

// hop 1, leader side: thread t adds the four wavefront words of slot t % 8 of member t / 8; the members of a
// wavefront are added across lanes, the four wavefronts through LDS.  Publishes the die's line and keeps its float32
// totals in xs.stage2[die][slot].  Returns false if the wait was abandoned.
template <class XS>
__device__ __forceinline__ bool tree8_die_totals(const PArgs& pa, unsigned int seq, XS& xs) {
    const int tid = threadIdx.x, x = pa.wg, p = tid & 7, mi = tid >> 3;
    const int nmem = (pa.G - x + DIES - 1) / DIES;
    const bool valid = mi >= 1 && mi < nmem;
    const unsigned long long* src = pa.buf1 + ((size_t)(seq & 1u) * PT + x + (size_t)mi * DIES) * 32 + p;
    unsigned long long w[4];
    bool aborted = false;
    if (valid) aborted = !poll_words<4>(pa, src, 8, seq, w);
    __syncthreads();  // the wavefronts' stores to xs.own lie before this barrier
    double s = 0.0;
    if (valid)
        s = ((double)__uint_as_float((unsigned int)w[0]) + (double)__uint_as_float((unsigned int)w[1])) +
            ((double)__uint_as_float((unsigned int)w[2]) + (double)__uint_as_float((unsigned int)w[3]));
    else if (mi == 0)
        s = ((double)xs.own[p] + (double)xs.own[8 + p]) + ((double)xs.own[16 + p] + (double)xs.own[24 + p]);
    s = sum_over_lane_bits_3_to_5(s);  // the eight members of this wavefront
    if ((tid & 63) < 8) xs.red2[(tid >> 6) * 8 + p] = s;
    if (aborted) {
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (xs.abort) return false;
    if (tid < 8) {
        const float tot = (float)((xs.red2[tid] + xs.red2[8 + tid]) + (xs.red2[16 + tid] + xs.red2[24 + tid]));
        xs.stage2[x * 8 + tid] = tot;
        st_word(&pa.buf3[((size_t)(seq & 1u) * DIES + x) * 32 + tid], pack_f(seq, tot));
    }
    return true;
}

// hop 2 inside wavefront 0 (the other wavefronts go straight to the caller's barrier): lane 8 x + p waits for slot p
// of die x; the eight dies are added across lanes; the grid totals go to xs.totd[accumulator].  A leader's own die
// is read from xs.stage2.  On an abandoned wait xs.abort is set.  No barrier inside.
template <int NACC, class XS>
__device__ __forceinline__ void tree8_grid_totals_wave0(const PArgs& pa, unsigned int seq, XS& xs) {
    const int lane = threadIdx.x, x = lane >> 3, p = lane & 7;
    const unsigned long long* src = pa.buf3 + ((size_t)(seq & 1u) * DIES + x) * 32 + p;
    unsigned long long w[1];
    double s;
    wave_lds_sync();  // (a leader's lanes 0 .. 7 have just written its own die's totals)
    if (x == pa.wg) {
        s = (double)xs.stage2[x * 8 + p];
    } else if (HOP2_PIPE > 1 ? poll_word_staggered<HOP2_PIPE, HOP2_SLEEP>(pa, src, seq, w[0]) : poll_words<1>(pa, src, 0, seq, w)) {
        s = (double)__uint_as_float((unsigned int)w[0]);
    } else {
        s = 0.0;
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    s = sum_over_lane_bits_3_to_5(s);
    if (lane < 8 && slot_acc(p) < NACC) xs.totd[slot_acc(p)] = s;
    wave_lds_sync();  // the caller's lanes read one another's totals
}

// The same hop for the loops (forward evaluations, (dF/dC)^T passes): the totals stay in registers -- every lane l
// returns the grid total of slot l % 8, i.e. of accumulator slot_acc(l % 8) -- and an abandoned wait is reported by the
// return value (the same in all lanes), so that nothing between the arrival of the totals and the update waits for LDS.
// All 64 lanes of wavefront 0 call it.
template <class XS>
__device__ __forceinline__ bool tree8_grid_totals_regs(const PArgs& pa, unsigned int seq, XS& xs, double& total) {
    const int lane = threadIdx.x, x = lane >> 3, p = lane & 7;
    const unsigned long long* src = pa.buf3 + ((size_t)(seq & 1u) * DIES + x) * 32 + p;
    unsigned long long w[1];
    double s;
    bool failed = false;
    wave_lds_sync();  // (a leader's lanes 0 .. 7 have just written its own die's totals)
    if (x == pa.wg) {
        s = (double)xs.stage2[x * 8 + p];
    } else if (HOP2_PIPE > 1 ? poll_word_staggered<HOP2_PIPE, HOP2_SLEEP>(pa, src, seq, w[0]) : poll_words<1>(pa, src, 0, seq, w)) {
        s = (double)__uint_as_float((unsigned int)w[0]);
    } else {
        s = 0.0;
        failed = true;
        xs.abort = 1;
        __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    total = sum_over_lane_bits_3_to_5(s);
    return __builtin_amdgcn_ballot_w64(failed) == 0ull;
}
// Total of accumulator a (a < 8, any value per lane) from the registers tree8_grid_totals_regs left: all 64 lanes call it.
__device__ __forceinline__ double tree8_total_of(double total, int a) {
    const int src = slot_acc(a & 7) << 2;
    return __hiloint2double(__builtin_amdgcn_ds_bpermute(src, __double2hiint(total)),
                            __builtin_amdgcn_ds_bpermute(src, __double2loint(total)));
}

// Both hops after publish_partials: grid totals of the NACC sums in xs.totd, in every workgroup; ends with a barrier.
template <int NACC, class XS>
__device__ __forceinline__ bool tree_totals(const PArgs& pa, unsigned int seq, XS& xs) {
    if constexpr (NACC <= WAVE_WORDS_MAX) {
        if (pa.wg < DIES && !tree8_die_totals(pa, seq, xs)) return false;
        if (threadIdx.x < 64) tree8_grid_totals_wave0<NACC>(pa, seq, xs);
        __syncthreads();
        return xs.abort == 0;
    } else {
        if (pa.wg < DIES && !tree_die_totals<NACC>(pa, seq, xs)) return false;
        return tree_grid_totals<NACC>(pa, seq, xs);
    }
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));

// One pass over the workgroup's LDS tile.
// SHARED: the workgroup shares its SIMDs with other teams' workgroups (batched launches); the hardware then
// interleaves wavefronts, and short groups keep the registers low enough for four or five workgroups per compute unit.
// s_tab: the caller's LDS table of the product forms' per-codeword operands (fwd_dot_tables), or null: then every lane
// forms them itself in prepare().
template <int K, int D, int DIST, int PASS, bool SHARED>
__device__ __forceinline__ void tile_pass(const Args& a, const float* s_w, const float* s_g, int64_t base, int cnt,
                                          const float* s_Cf, const float* s_Hs, const float* s_Ff,
                                          float (&acc)[SmallItem<K, D, DIST, PASS>::NREG], const float* s_tab = nullptr) {
    using Item = SmallItem<K, D, DIST, PASS>;
    float c[K][D], hs[K][D], ff[K][D + 1];
#pragma unroll
    for (int j = 0; j < K; ++j)
#pragma unroll
        for (int r = 0; r < D; ++r) {
            c[j][r] = s_Cf[j * D + r];
            hs[j][r] = Item::USE_H ? s_Hs[j * D + r] : 0.f;
            ff[j][r] = Item::USE_F ? s_Ff[j * D + r] : 0.f;
        }
    if constexpr (Item::FWD_DOT || Item::B2_DOT) {
        // the per-codeword operands of the product form: from the caller's LDS table where it keeps one (formed once per
        // evaluation by wavefront 0), else formed here by every lane
        if (s_tab) {
#pragma unroll
            for (int j = 0; j < K; ++j) {
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    if (Item::FWD_DOT)
                        hs[j][r] = s_tab[j * D + r];
                    else
                        c[j][r] = s_tab[j * D + r];
                }
                ff[j][Item::FWD_DOT ? 0 : D] = s_tab[K * D + j];
                if (Item::B2_DOT) ff[j][0] = s_tab[K * D + K + D + j];
            }
#pragma unroll
            for (int r = 0; r < D; ++r) ff[r][1] = s_tab[K * D + K + r];
        } else {
            Item::prepare(a, c, hs, ff);
        }
    } else {
        Item::prepare(a, c, hs, ff);
    }
    if constexpr (Item::FOLD_HF || (Item::B2_DOT && K * D >= 32)) {
        // the codebook is the same for all lanes: as scalar registers it leaves the vector registers to h and the sums
#pragma unroll
        for (int j = 0; j < K; ++j)
#pragma unroll
            for (int r = 0; r < D; ++r) c[j][r] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, c[j][r])));
    }
#pragma unroll
    for (int q = 0; q < Item::NREG; ++q) acc[q] = 0.f;
    // one wavefront per SIMD: the latencies of a vector's chain (LDS load, exponentials, reciprocal) are hidden by
    // other vectors of the same lane, so vectors are taken in groups whose bodies the scheduler interleaves: in the
    // forward passes groups of UNR while they last, then groups of 4, then single vectors
    constexpr bool FWD_LIKE = (PASS == PASS_FWD || PASS == PASS_FIN);
    // (for k = 8 and 16 the group size makes no measurable difference: 2 to 16 vectors are within 2 % of each other;
    // in the backward passes at k <= 4, 4 / 6 / 9 / 12 vectors give 6.53 / 6.34 / 6.30 / 6.24 us per pass at C3; in the forward
    // loop 9 / 12 / 18 / 36 give 4.79 / 4.79 / 4.71 / 4.65 us per evaluation)
#ifndef IDKM_FWD_UNR
#define IDKM_FWD_UNR 18
#endif
#ifndef IDKM_BWD_UNR
#define IDKM_BWD_UNR 12
#endif
    constexpr int UNR = SHARED ? (K <= 4 ? 4 : 2)
                               : (FWD_LIKE ? (K <= 4 ? IDKM_FWD_UNR : (K == 8 ? 8 : 4)) : (K <= 4 ? IDKM_BWD_UNR : (K == 8 ? 3 : 2)));
    auto one = [&](int it) {
        float w[D], g[D];
#pragma unroll
        for (int r = 0; r < D; ++r) {
            w[r] = s_w[it * D + r];
            g[r] = Item::USE_G ? s_g[it * D + r] : 0.f;
        }
        Item::run(a, base + it, w, g, c, hs, ff, acc);
    };
    if constexpr (FWD_LIKE) {
        int it = threadIdx.x;
        if constexpr (UNR >= 18) {
            // a tile of 2 UNR or more vectors per lane: one straight block of 2 UNR bodies first (C3: the whole tile)
            for (; it + (2 * UNR - 1) * PT < cnt; it += 2 * UNR * PT) {
#pragma unroll
                for (int u = 0; u < 2 * UNR; ++u) one(it + u * PT);
            }
        }
        for (; it + (UNR - 1) * PT < cnt; it += UNR * PT) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) one(it + u * PT);
        }
        if (UNR > 4) {
            for (; it + 3 * PT < cnt; it += 4 * PT) {
#pragma unroll
                for (int u = 0; u < 4; ++u) one(it + u * PT);
            }
        }
        for (; it < cnt; it += PT) one(it);
    } else if constexpr (PASS == PASS_B2 && K <= 4 && D == 1 && !SHARED) {
        // the pass an implicit solve repeats, scalar weights: straight blocks of 36 vectors per lane while they last (C3:
        // the whole tile), then of UNR, of 4, and single vectors (6.29 -> 6.06 us per pass at C3 against blocks of 12)
        int it = threadIdx.x;
        for (; it + 35 * PT < cnt; it += 36 * PT) {
#pragma unroll
            for (int u = 0; u < 36; ++u) one(it + u * PT);
        }
        for (; it + (UNR - 1) * PT < cnt; it += UNR * PT) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) one(it + u * PT);
        }
        for (; it + 3 * PT < cnt; it += 4 * PT) {
#pragma unroll
            for (int u = 0; u < 4; ++u) one(it + u * PT);
        }
        for (; it < cnt; it += PT) one(it);
    } else {
        // the backward passes carry more state per vector; a plainly unrolled loop schedules them better (measured)
#pragma unroll UNR
        for (int it = threadIdx.x; it < cnt; it += PT) one(it);
    }
    Item::finish(a, c, acc);
}

// The same pass for a layer that does not fit the chip's LDS: W (and dL/dWq) are read from memory in every pass, 16
// bytes per lane and load, with the loads of the next batch in flight while the current one is worked on (one
// wavefront per SIMD has nothing else to hide their latency with).  The workgroups of the team take 4 KB blocks in
// turn (block t G + wg in round t), so that at any moment the team reads one contiguous window of memory: with a
// contiguous share per workgroup and a power-of-two layer, all workgroups would hit the same memory channel.
// gw, gg: the whole tensors, 16-byte aligned.
template <int K, int D, int DIST, int PASS>
__device__ __forceinline__ void tile_pass_global(const Args& a, const float* gw, const float* gg, int wg, int G,
                                                 const float* s_Cf, const float* s_Hs, const float* s_Ff,
                                                 float (&acc)[SmallItem<K, D, DIST, PASS>::NREG]) {
    using Item = SmallItem<K, D, DIST, PASS>;
    float c[K][D], hs[K][D], ff[K][D + 1];
#pragma unroll
    for (int j = 0; j < K; ++j)
#pragma unroll
        for (int r = 0; r < D; ++r) {
            c[j][r] = s_Cf[j * D + r];
            hs[j][r] = Item::USE_H ? s_Hs[j * D + r] : 0.f;
            ff[j][r] = Item::USE_F ? s_Ff[j * D + r] : 0.f;
        }
    Item::prepare(a, c, hs, ff);
#pragma unroll
    for (int q = 0; q < Item::NREG; ++q) acc[q] = 0.f;
    constexpr int VPL = 4 / D;                // vectors per 16-byte load
    constexpr int NLD = Item::USE_G ? 4 : 8;  // loads in flight per lane and operand
    const int64_t ngroups = a.m / VPL;        // whole 16-byte groups of the layer
    const f32x4_t* w4 = reinterpret_cast<const f32x4_t*>(gw);
    const f32x4_t* g4 = reinterpret_cast<const f32x4_t*>(gg);
    auto work = [&](int64_t gi, const f32x4_t& wq, const f32x4_t& gq) {
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            float w[D], g[D];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                w[r] = wq[v * D + r];
                g[r] = Item::USE_G ? gq[v * D + r] : 0.f;
            }
            Item::run(a, gi * VPL + v, w, g, c, hs, ff, acc);
        }
    };
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    f32x4_t cw[NLD], cg[NLD], nw[NLD], ng[NLD];
    const int64_t step = (int64_t)G * PT;           // groups per round of the team
    int64_t gi = (int64_t)wg * PT + threadIdx.x;    // this lane's group on its first turn
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
        const int64_t i = gi + u * step;
        cw[u] = (i < ngroups) ? w4[i] : zero;
        cg[u] = (Item::USE_G && i < ngroups) ? g4[i] : zero;
    }
    // the loop bound is the same for all lanes of the workgroup up to the last, partial block
    for (; gi < ngroups; gi += NLD * step) {
        const int64_t nx = gi + NLD * step;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int64_t i = nx + u * step;
            nw[u] = (i < ngroups) ? w4[i] : zero;
            ng[u] = (Item::USE_G && i < ngroups) ? g4[i] : zero;
        }
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            if (gi + u * step < ngroups) work(gi + u * step, cw[u], cg[u]);
        }
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            cw[u] = nw[u];
            cg[u] = ng[u];
        }
    }
    // the vectors behind the last whole 16-byte group of the layer (fewer than VPL) go to the last workgroup
    if (wg == G - 1) {
        for (int64_t it = ngroups * VPL + threadIdx.x; it < a.m; it += PT) {
            float w[D], g[D];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                w[r] = gw[it * D + r];
                g[r] = Item::USE_G ? gg[it * D + r] : 0.f;
            }
            Item::run(a, it, w, g, c, hs, ff, acc);
        }
    }
    Item::finish(a, c, acc);
}

// A pass over the workgroup's share of the layer: its LDS tile (w, g: the tile; base, cnt: its place in the layer) or,
// GLOBALW, its blocks of the tensors in memory (w, g: the whole tensors).
template <int K, int D, int DIST, int PASS, bool SHARED, bool GLOBALW>
__device__ __forceinline__ void any_tile_pass(const Args& a, const PArgs& pa, const float* w, const float* g,
                                              int64_t base, int cnt, const float* s_Cf, const float* s_Hs,
                                              const float* s_Ff, float (&acc)[SmallItem<K, D, DIST, PASS>::NREG],
                                              const float* s_tab = nullptr) {
    if constexpr (GLOBALW)
        tile_pass_global<K, D, DIST, PASS>(a, w, g, pa.wg, pa.G, s_Cf, s_Hs, s_Ff, acc);
    else
        tile_pass<K, D, DIST, PASS, SHARED>(a, w, g, base, cnt, s_Cf, s_Hs, s_Ff, acc, s_tab);
}

// Codewords per reducer: as many as fit 8 words of (n_j, s_j) per workgroup.
constexpr int cw_per_reducer(int K, int D) {
    int kpr = 8 / (D + 1);
    if (kpr < 1) kpr = 1;
    int p = 1;
    while (p * 2 <= kpr) p *= 2;
    return p > K ? K : p;
}

// Operands of the product form of the forward loop (SmallItem::FWD_DOT), formed once per evaluation by wavefront 0
// (all 64 lanes call; lane j d + r < k d passes component r of codeword j, the other lanes zero) instead of by every lane
// at the start of its pass:  tab[j d + r] = ascale (c_jr - mu_r) (ascale = 2 s^2), tab[k d + j] = -s^2 |c_j - mu|^2, tab[k d + k + r] = mu_r,
// mu the mean codeword.  The sums over codewords and over components run across the lanes.
template <int K, int D>
__device__ __forceinline__ float fwd_dot_tables(float c, float s2, float* tab, float ascale) {
    static_assert(D == 2 || D == 4, "lane layout j d + r with d a divisor of 4");
    const int lane = threadIdx.x;
    // mu_r: over the lanes with the same lane % d
    float m = c;
    if (D == 2) m += dpp_f<0x4E, 0xf>(0.f, m);  // quad_perm [2,3,0,1]
    m += dpp_f<0x124, 0xf>(0.f, m);              // row_ror:4
    m += dpp_f<0x128, 0xf>(0.f, m);              // row_ror:8
    m = cross_row_sum(m) * (1.f / K);
    const float dc = c - m;
    // |c_j - mu|^2: over the d lanes of codeword j
    float q = dc * dc;
    q += dpp_f<0xB1, 0xf>(0.f, q);               // quad_perm [1,0,3,2]
    if (D == 4) q += dpp_f<0x4E, 0xf>(0.f, q);
    if (lane < K * D) {
        tab[lane] = ascale * dc;
        if (lane % D == 0) tab[K * D + lane / D] = -s2 * q;
        if (lane < D) tab[K * D + K + lane] = m;
    }
    return m;  // mu_r of this lane's component
}
// The backward's table keeps c_j - mu itself (ascale = 1) and, behind mu, h_j . (F*_j - mu) / tau of the current h:
// lane j d + r passes h_jr / tau times (F*_jr - mu_r); the d lanes of a codeword are added across lanes.
template <int K, int D>
__device__ __forceinline__ void bwd_dot_hf(float hfm, float* tab) {
    const int lane = threadIdx.x;
    hfm += dpp_f<0xB1, 0xf>(0.f, hfm);              // quad_perm [1,0,3,2]
    if (D == 4) hfm += dpp_f<0x4E, 0xf>(0.f, hfm);  // quad_perm [2,3,0,1]
    if (lane < K * D && lane % D == 0) tab[K * D + K + D + lane / D] = hfm;
}

// Forward solve (Alg. 1) and the evaluation at C*, in one launch.
// GLOBALW: the layer does not fit the chip's LDS; every pass reads the workgroup's share of W from memory.
template <int K, int D, int DIST, bool SHARED, bool GLOBALW = false>
__device__ __forceinline__ void persist_fwd_body(const Args& a, const PArgs& pa) {
    constexpr int KD = K * D;
    constexpr int ACCW = D + 1;
    constexpr int NACC = K * ACCW;
    constexpr int KPR = cw_per_reducer(K, D);  // codewords owned by one reducer
    constexpr int R = K / KPR;                 // reducers
    constexpr int WPR = KPR * ACCW;            // words a reducer reads per workgroup
    constexpr int NB = KD;                     // broadcast words: the new codebook
    static_assert(NACC <= XLINE && NB <= XBCAST && KD <= 64 && PT / 16 == 16, "shape does not fit the exchange layout");
    extern __shared__ float s_tile[];
    __shared__ XShared<NACC> xs;
    __shared__ double s_Cd[KD];  // float64 master copy (a reducer's own slice is the live one)
    __shared__ float s_Cf[KD];
    __shared__ int s_done, s_iters, s_conv, s_bad;
    __shared__ double s_res;
    // product form of the loop's E-step: its per-codeword operands, kept up to date by wavefront 0
    // (worth it from k d = 32 on: below, what a lane saves at the start of its pass is less than wavefront 0 adds to the
    // path every workgroup waits on: k = 4, d = 2 4.38 -> 4.64 us per evaluation with the table, k = 16, d = 4 8.65 -> 8.39)
    constexpr bool DOT = SmallItem<K, D, DIST, PASS_FWD>::FWD_DOT && !GLOBALW && K * D >= 32;
    __shared__ float s_tab[DOT ? KD + K + D : 1];

    const int tid = threadIdx.x, wg = pa.wg;
    const int64_t base = (int64_t)wg * pa.per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < pa.per) ? (int)(a.m - base) : pa.per;
    tree_announce(pa);
    if (!GLOBALW)
        load_tile<PT>(s_tile, a.W + base * D, cnt * D);
    const float* s_w = GLOBALW ? a.W : s_tile;
    if (tid < KD) {
        const float c0 = pa.C0[tid];
        s_Cd[tid] = (double)c0;
        s_Cf[tid] = c0;
    }
    if (tid == 0) {
        xs.abort = 0;
        s_done = 0;
        s_iters = 0;
        s_conv = 0;
        s_bad = 0;
        s_res = 0.0;
    }
    if constexpr (DOT) {
        if (tid < 64) fwd_dot_tables<K, D>(tid < KD ? pa.C0[tid] : 0.f, -a.nscale, s_tab, -2.f * a.nscale);
    }
    __syncthreads();
    const double tol = pa.tol;
    const int max_iter = pa.max_iter;
    if (pa.tree && !tree_handshake(pa, xs)) return;
    // reducer r is workgroup r; with fewer than R workgroups the first ones take several slices in turn
    unsigned int seq = pa.seq_base;

    int r_iters = 0;
    // Centre update of the whole codebook (Alg. 1) and the stop test from grid totals every workgroup holds (a team
    // of one, or the two-level exchange): tot(i) is total i of the K (D+1) sums.  Wavefront 0; lane 0 decides.
    // (lanes < k d of wavefront 0 keep their component of the codebook in registers too: float64 master and float32 copy)
    double r_cd = 0.0;
    float r_cf = 0.f;
    if (tid < KD) {
        r_cf = pa.C0[tid];
        r_cd = (double)r_cf;
    }
    // n, sv: mass of this lane's codeword and the sum of its component (lanes < k d; all 64 lanes of wavefront 0 call)
    auto update_vals = [&](double n, double sv) {
        double df2 = 0.0;
        if (tid < KD) {
            double cnew = (n > 0.0) ? fast_div_d(sv, n) : r_cd;
            if (!(n >= 0.0) || !(fabs(sv) <= 1.7e308) || !(fabs(cnew) <= 1.7e308)) cnew = __builtin_nan("");
            r_cd = cnew;
            s_Cd[tid] = cnew;
            const float cn = (float)cnew;
            const double df = (double)cn - (double)r_cf;
            df2 = df * df;
            r_cf = cn;
            s_Cf[tid] = cn;
        }
        const double r2 = first_lanes_sum_d_dpp<KD>(df2);
        r_iters += 1;  // (wavefront 0 counts in a register: nothing on this path waits for an LDS read of the state)
        if (tid == 0) {
            s_iters = r_iters;
            s_res = r2;  // squared; the root is taken once, when the solve is over
            const bool bad = !(r2 <= 1.7e308);
            if (bad) s_bad = 1;
            const bool conv = r2 < tol * tol;
            s_conv = conv ? 1 : 0;
            if (conv || bad || r_iters >= max_iter) s_done = 1;
        }
    };
    auto update_all = [&](auto tot) {
        double n = 0.0, sv = 0.0;
        if (tid < KD) {
            const int j = tid / D, rr = tid - j * D;
            n = tot(j * ACCW);
            sv = tot(j * ACCW + 1 + rr);
        }
        update_vals(n, sv);
    };

    float acc[NACC];
    while (!s_done) {
        IDKM_STAMP(0);
        any_tile_pass<K, D, DIST, PASS_FWD, SHARED, GLOBALW>(a, pa, s_w, nullptr, base, cnt, s_Cf, nullptr, nullptr, acc, DOT ? s_tab : nullptr);
        IDKM_STAMP(1);
        ++seq;
        publish_partials<NACC>(pa, seq, acc, xs);
        IDKM_STAMP(2);
        if (pa.G == 1) {
            // a team of one has no exchange: its partial sums (xs.own, the float32 words it would have published)
            // are the totals, and the whole codebook is updated here
            __syncthreads();
            if (tid < 64) update_all([&](int i) { return (double)xs.own[i]; });
        } else if (pa.tree) {
            if constexpr (NACC <= WAVE_WORDS_MAX) {
                // hop 2 and the update stay inside wavefront 0: no barrier between them
                if (wg < DIES) {
                    if (!tree8_die_totals(pa, seq, xs)) return;
                    IDKM_STAMP(3);
                }
                if (tid < 64) {
                    double total;
                    const bool ok = tree8_grid_totals_regs(pa, seq, xs, total);
                    IDKM_STAMP(4);
                    const int jj = (tid < KD) ? tid / D : 0, rr = (tid < KD) ? tid - jj * D : 0;
                    const double n = tree8_total_of(total, jj * ACCW), sv = tree8_total_of(total, jj * ACCW + 1 + rr);
                    if (ok) update_vals(n, sv);
                }
            } else {
                if (!tree_totals<NACC>(pa, seq, xs)) return;
                IDKM_STAMP(4);
                if (tid < 64) update_all([&](int i) { return xs.totd[i]; });
            }
        } else {
        for (int r = wg; r < R; r += pa.G) {
            if (!reduce_slice<NACC, WPR>(pa, seq, r * WPR, xs)) return;
            IDKM_STAMP(3);
#ifdef IDKM_TRACE
            if (pa.trace && threadIdx.x == 0 && pa.wg == 0 && s_iters < 64) pa.trace[s_iters * 8 + 6] = pa.trace[2 * 64 * 8 - 1];
#endif
            // centre update of this slice (Alg. 1), float64; a non-finite sum is broadcast as NaN
            if (tid < KPR * D) {
                const int jl = tid / D, rr = tid - jl * D, idx = (r * KPR + jl) * D + rr;
                const double n = xs.tot[jl * ACCW], s = xs.tot[jl * ACCW + 1 + rr];
                const double cold = s_Cd[idx];
                double cnew = (n > 0.0) ? fast_div_d(s, n) : cold;
                if (!(n >= 0.0) || !(fabs(s) <= 1.7e308) || !(fabs(cnew) <= 1.7e308)) cnew = __builtin_nan("");
                s_Cd[idx] = cnew;
                st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + idx], pack_f(seq, (float)cnew));
            }
            IDKM_SUB(8);
        }
        IDKM_STAMP(4);
        // hop 2 and the stop test, all inside wavefront 0: lane q waits for codeword component q, the squared
        // step ||C+ - C||_F^2 is formed from the float32 codebooks every workgroup holds (the same words through
        // the same DPP network, hence the same decision everywhere), lane 0 decides; one barrier publishes it.
        if (tid < 64) {
            double df2 = 0.0;
            bool aborted = false;
            if (tid < KD) {
                const unsigned long long* src = pa.buf2 + (size_t)(seq & 1u) * XBCAST + tid;
                unsigned long long w[1];
                float cn = 0.f;
                // a slice this workgroup reduced itself is taken from its own copy (the same float32 value it
                // has just broadcast): the reducer, which every other workgroup waits for, does not wait for the
                // round trip of its own store
                const bool own = ((tid / (KPR * D)) % pa.G) == wg;
                if (own)
                    cn = (float)s_Cd[tid];
                else if (poll_words<1>(pa, src, 0, seq, w))
                    cn = __uint_as_float((unsigned int)w[0]);
                else
                    aborted = true;
                const double df = (double)cn - (double)s_Cf[tid];
                df2 = df * df;
                s_Cf[tid] = cn;
            }
            if (aborted) {
                xs.abort = 1;
                __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            IDKM_SUB(9);
            const double r2 = first_lanes_sum_d_dpp<KD>(df2);  // lanes >= KD hold zero; lane 0 decides
            if (tid == 0) {
                s_iters += 1;
                s_res = r2;  // squared; the root is taken once, when the solve is over
                const bool bad = !(r2 <= 1.7e308);
                if (bad) s_bad = 1;
                const bool conv = r2 < tol * tol;
                s_conv = conv ? 1 : 0;
                if (conv || bad || s_iters >= max_iter) s_done = 1;
            }
        }
        }
        if constexpr (DOT) {
            if (tid < 64) {  // (wavefront 0 has just written the new codebook)
                wave_lds_sync();
                fwd_dot_tables<K, D>(tid < KD ? s_Cf[tid] : 0.f, -a.nscale, s_tab, -2.f * a.nscale);
            }
        }
        __syncthreads();
        IDKM_SUB(10);
        if (xs.abort) return;
        IDKM_STAMP(5);
    }

    // evaluation at C*: outputs, and n*, F* for the backward
    any_tile_pass<K, D, DIST, PASS_FIN, SHARED, GLOBALW>(a, pa, s_w, nullptr, base, cnt, s_Cf, nullptr, nullptr, acc);
    ++seq;
    publish_partials<NACC>(pa, seq, acc, xs);
    if (pa.tree) {
        // only workgroup 0 needs these totals: it writes the state and, last, the word that says the launch ran to
        // its end; the other leaders add up their die and leave, everybody else has left already
        if constexpr (NACC <= WAVE_WORDS_MAX) {
            if (wg < DIES && !tree8_die_totals(pa, seq, xs)) return;
            if (wg != 0) return;
            if (tid < 64) tree8_grid_totals_wave0<NACC>(pa, seq, xs);
            __syncthreads();
            if (xs.abort) return;
        } else {
            if (wg < DIES && !tree_die_totals<NACC>(pa, seq, xs)) return;
            if (wg != 0) return;
            if (!tree_grid_totals<NACC>(pa, seq, xs)) return;
        }
        {
            if (tid < KD) {
                const int j = tid / D, rr = tid - j * D;
                const double n = xs.totd[j * ACCW], s = xs.totd[j * ACCW + 1 + rr];
                const double cst = (double)s_Cf[tid];
                const double f = (n > 0.0) ? fast_div_d(s, n) : cst;
                a.Cd[tid] = cst;
                a.Cf[tid] = s_Cf[tid];
                a.Fd[tid] = f;
                a.Ff[tid] = (float)f;
                if (rr == 0) a.nd[j] = n;
                if (a.C_out) a.C_out[tid] = s_Cf[tid];
            }
            if (tid == 0) {
                int empty = 0, bad = 0;
                for (int j = 0; j < K; ++j) {
                    const double n = xs.totd[j * ACCW];
                    if (!(n > 0.0)) empty++;
                    if (!(n >= 0.0)) bad = 1;
                    for (int rr = 0; rr < D; ++rr)
                        if (!(fabs(xs.totd[j * ACCW + 1 + rr]) <= 1.7e308)) bad = 1;
                }
                PResult* o = pa.out;
                o->empty[0] = empty;
                o->bad[0] = bad;
                o->nred = 0;
                o->iters = s_iters;
                o->residual = sqrt(s_res);
                o->converged = s_conv;
                o->nonfinite = s_bad;
                o->done = pa.seq_base + 1u;
            }
        }
        return;
    }
    for (int r = wg; r < R; r += pa.G) {
        if (!reduce_slice<NACC, WPR>(pa, seq, r * WPR, xs)) return;
        if (tid < KPR * D) {
            const int jl = tid / D, rr = tid - jl * D, j = r * KPR + jl, idx = j * D + rr;
            const double n = xs.tot[jl * ACCW], s = xs.tot[jl * ACCW + 1 + rr];
            const double cst = (double)s_Cf[idx];
            const double f = (n > 0.0) ? fast_div_d(s, n) : cst;
            a.Cd[idx] = cst;
            a.Cf[idx] = s_Cf[idx];
            a.Fd[idx] = f;
            a.Ff[idx] = (float)f;
            if (rr == 0) a.nd[j] = n;
            if (a.C_out) a.C_out[idx] = s_Cf[idx];
        }
        if (tid == 0) {
            int empty = 0, bad = 0;
            for (int jl = 0; jl < KPR; ++jl) {
                const double n = xs.tot[jl * ACCW];
                if (!(n > 0.0)) empty++;
                if (!(n >= 0.0)) bad = 1;
                for (int rr = 0; rr < D; ++rr)
                    if (!(fabs(xs.tot[jl * ACCW + 1 + rr]) <= 1.7e308)) bad = 1;
            }
            pa.out->empty[r] = empty;
            pa.out->bad[r] = bad;
            // this reducer's slice of the state is written: the host takes the launch as complete only when every
            // reducer has said so (a reducer that gives up its wait in this last stage never does)
            pa.out->fin[r] = pa.seq_base + 1u;
        }
        __syncthreads();
    }
    if (wg == pa.G - 1 && tid == 0) {
        PResult* o = pa.out;
        o->nred = R;
        o->iters = s_iters;
        o->residual = sqrt(s_res);
        o->converged = s_conv;
        o->nonfinite = s_bad;
        o->done = pa.seq_base + 1u;
    }
}

// State of the minimal-residual (restarted GMRES) solve of (I - dF/dC*)^T g = v inside the persistent backward: every
// workgroup of a team that receives the grid totals (a team of one, or the two-level exchange) keeps the whole of it
// and takes every step itself, in float64, so that all workgroups hold the same iterate.  N = k d <= 64 unknowns, a
// basis of R <= N vectors; the arrays lie in the launch's dynamic LDS behind the tiles (at k d = 64, R = 64 they are
// 67 KB, which only calls of this mode pay for).
__host__ __device__ constexpr size_t gm_state_doubles(int n, int r) {
    // Q, H, cs, sn, sv, y, p, w, beta
    return (size_t)(r + 1) * (n + 1) + (size_t)r * (r + 1) + r + r + (r + 1) + r + (r + 1) + n + 1;
}
__host__ __device__ constexpr size_t gm_state_bytes(int n, int r) { return gm_state_doubles(n, r) * sizeof(double) + 16; }
__host__ __device__ constexpr int gm_basis_length(int asked, int n) { return asked < n ? (asked < 1 ? 1 : asked) : n; }

template <int N>
struct GmView {
    static constexpr int QS = N + 1;  // row stride of Q: lanes that read one row each then fall on different LDS banks
    double* Q;    // [R + 1][QS] orthonormal basis, row i = q_i
    double* H;    // [R][R + 1] Hessenberg columns, rotated in place to triangular
    double *cs, *sn, *sv, *y, *p, *w, *beta;
    int* ctl;     // phase, j, stall
    int R, HS;
    __device__ __forceinline__ void bind(void* mem, int r) {
        R = r;
        HS = r + 1;
        double* d = reinterpret_cast<double*>(mem);
        Q = d;   d += (size_t)(r + 1) * QS;
        H = d;   d += (size_t)r * (r + 1);
        cs = d;  d += r;
        sn = d;  d += r;
        sv = d;  d += r + 1;
        y = d;   d += r;
        p = d;   d += r + 1;
        w = d;   d += N;
        beta = d; d += 1;
        ctl = reinterpret_cast<int*>(d);
    }
};

// One step of that solve in wavefront 0 (all 64 lanes call it; lanes idx < N own element idx).  u(idx) = the grid
// total of this pass: (dF/dC)^T applied to the vector the pass was run with -- basis vector q_j in phase 0, the
// iterate g in phase 1.  Same steps, stop rule and counting as the stream path's pass tail: classical Gram-Schmidt
// twice, Givens update of the least-squares problem, at the end of a cycle g += Q y and one pass for the true
// residual r = v + (dF/dC)^T g - g, whose norm is held to tol ||v||.  Leaves the next pass's vector in hnext (lanes
// < N; times 1/(tau n) and rounded to float32 by the caller) and returns 1 if the solve is over, else 0.
// Lane 0 writes the result fields through the references.
template <int N, class U>
__device__ __forceinline__ int gmres_step(const GmView<N>& gm, U u, const double* s_v, double* s_g, double tol, double vnorm,
                                         int max_iter, int& s_iters, int& s_conv, int& s_bad, double& s_res,
                                         double& hnext) {
    static_assert(N <= 64, "one lane per unknown and per basis vector");
    constexpr int QS = GmView<N>::QS;
    const int lane = threadIdx.x;
    wave_lds_sync();
    const int R = gm.R, HS = gm.HS;
    const int phase = __builtin_amdgcn_readfirstlane(gm.ctl[0]);
    int over = 0;
    hnext = 0.0;
    if (phase == 0) {
        const int j = __builtin_amdgcn_readfirstlane(gm.ctl[1]);
        double* hcol = gm.H + (size_t)j * HS;
        if (lane < N) gm.w[lane] = gm.Q[j * QS + lane] - u(lane);
        wave_lds_sync();
        double x = 0.0;
        for (int round = 0; round < 2; ++round) {
            // lane i <= j: h_i = q_i . w (its own row, element by element); then lane idx: w -= sum_i h_i q_i
            if (lane <= j) {
                const double* row = gm.Q + lane * QS;
                double pr = 0.0;
#pragma unroll 8
                for (int idx = 0; idx < N; ++idx) pr += row[idx] * gm.w[idx];
                gm.p[lane] = pr;
                hcol[lane] = round ? hcol[lane] + pr : pr;
            }
            wave_lds_sync();
            if (lane < N) {
                x = gm.w[lane];
#pragma unroll 4
                for (int i = 0; i <= j; ++i) x -= gm.p[i] * gm.Q[i * QS + lane];
                gm.w[lane] = x;
            }
            wave_lds_sync();
        }
        // |w|^2 across the lanes (valid in lane 0)
        const double w2 = first_lanes_sum_d_dpp<N>(lane < N ? x * x : 0.0);
        int next = 0;  // 0 next basis vector, 1 cycle over: apply to g, 3 done
        int nj_new = 0;
        double scale = 0.0;
        if (lane == 0) {
            const double hn = fast_sqrt_d(w2);
            // the earlier rotations on the new column; the running element stays in a register
            double hi = hcol[0];
            for (int i = 0; i < j; ++i) {
                const double h1 = hcol[i + 1], c = gm.cs[i], sn = gm.sn[i];
                hcol[i] = c * hi + sn * h1;
                hi = -sn * hi + c * h1;
            }
            const double hj = hi;
            const double rr = fast_sqrt_d(hj * hj + hn * hn);
            const double irr = rr > 0.0 ? fast_rcp_d(rr) : 0.0;
            const double cj = rr > 0.0 ? hj * irr : 1.0, sj = hn * irr;
            gm.cs[j] = cj;
            gm.sn[j] = sj;
            hcol[j] = rr;
            const double svj = gm.sv[j];
            gm.sv[j + 1] = -sj * svj;
            gm.sv[j] = cj * svj;
            const double est = fabs(sj * svj);
            s_iters += 1;
            s_res = est * est;
            const bool finite = (w2 <= 1.7e308) && (rr <= 1.7e308);
            const bool vanished = !(hn > 1e-14 * rr);
            const bool last = (j + 1 >= R) || (s_iters + 1 >= max_iter);
            if (!finite) {
                s_bad = 1;
                next = 3;
            } else if (vanished || last || est <= 0.5 * tol * vnorm) {
                nj_new = (rr > 0.0) ? j + 1 : j;
                gm.ctl[1] = nj_new;
                next = 1;
            } else {
                gm.ctl[1] = j + 1;
                scale = fast_rcp_d(hn);
            }
        }
        wave_lds_sync();
        // (what lane 0 decided travels in registers: the other lanes must not take their own stale view of the state)
        next = __builtin_amdgcn_readfirstlane(next);
        nj_new = __builtin_amdgcn_readfirstlane(nj_new);
        scale = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(scale)),
                                 __builtin_amdgcn_readfirstlane(__double2loint(scale)));
        if (next == 0) {
            if (lane < N) {
                const double q = x * scale;
                gm.Q[(j + 1) * QS + lane] = q;
                hnext = q;
            }
        } else if (next == 1) {
            const int nj = nj_new;
            // back substitution of the triangular system, one unknown per step: lane l holds the running right-hand
            // side of row l; y_i is taken from lane i and leaves every row above it
            double t = (lane < nj) ? gm.sv[lane] : 0.0;
            for (int i = nj - 1; i >= 0; --i) {
                const double ti = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(t), i),
                                                   __builtin_amdgcn_readlane(__double2loint(t), i));
                const double yi = ti * fast_rcp_d(gm.H[(size_t)i * HS + i]);
                if (lane < i) t -= gm.H[(size_t)i * HS + lane] * yi;
                if (lane == i) gm.y[i] = yi;
            }
            wave_lds_sync();
            if (lane < N) {
                double g = s_g[lane];
#pragma unroll 4
                for (int i = 0; i < nj; ++i) g += gm.y[i] * gm.Q[i * QS + lane];
                s_g[lane] = g;
                hnext = g;
            }
            if (lane == 0) gm.ctl[0] = 1;
        } else {
            over = 1;
        }
        return over;
    }
    // phase 1: true residual at g
    double r = 0.0;
    if (lane < N) r = s_v[lane] + u(lane) - s_g[lane];
    const double r2 = first_lanes_sum_d_dpp<N>(r * r);
    int next = 2;  // 2 new cycle from the residual, 3 done
    double scale = 0.0;
    if (lane == 0) {
        const double beta = fast_sqrt_d(r2);
        s_iters += 1;
        s_res = r2;
        if (!(r2 <= 1.7e308)) {
            s_bad = 1;
            next = 3;
        } else if (beta <= tol * vnorm) {
            s_conv = 1;
            next = 3;
        } else {
            gm.ctl[2] = (beta > 0.95 * gm.beta[0]) ? gm.ctl[2] + 1 : 0;
            if (gm.ctl[2] >= 2 || s_iters + 2 > max_iter) next = 3;
        }
        if (next == 2) {
            gm.beta[0] = beta;
            gm.ctl[0] = 0;
            gm.ctl[1] = 0;
            gm.sv[0] = beta;
            scale = fast_rcp_d(beta);
        }
    }
    wave_lds_sync();
    next = __builtin_amdgcn_readfirstlane(next);
    scale = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(scale)),
                             __builtin_amdgcn_readfirstlane(__double2loint(scale)));
    if (next == 2) {
        if (lane < N) {
            const double q = r * scale;
            gm.Q[lane] = q;
            hnext = q;
        }
        return 0;
    }
    // done: the caller keeps h(g)/tau from the end of the cycle for the final pass
    if (lane < N) hnext = s_g[lane];
    return 1;
}

// Backward (Alg. 2 per-layer steps): v, the averaged fixed-point iteration of
// Sec. 4.2 for g (skipped for JFB), and dW, in one launch.
template <int K, int D, int DIST, bool SHARED, bool GLOBALW = false>
__device__ __forceinline__ void persist_bwd_body(const Args& a, const PArgs& pa) {
    constexpr int KD = K * D;
    constexpr int KPR = (8 / D) > K ? K : (8 / D);  // codewords per reducer: 8 words of D components
    constexpr int R = K / KPR;
    constexpr int WPR = KPR * D;
    constexpr int NB = KD + R;  // broadcast words: h/tau, then one partial squared norm per reducer
    static_assert(KD <= XLINE && NB <= XBCAST && KD <= 64, "shape does not fit the exchange layout");
    // explicit-Jacobian mode (Eq. "grad", "inv" taken literally): offered when its K D (K D + D + 1) sums fit one
    // exchange line
    constexpr int NBJ = KD * KD + KD * D + KD;
    constexpr bool HAS_DENSE = NBJ <= XDENSE;
    extern __shared__ float s_tile[];
    __shared__ XShared<HAS_DENSE ? NBJ : KD> xs;
    __shared__ double s_v[KD], s_g[KD], s_rn[K];  // a reducer's own slice is the live one; s_rn = 1/(tau n)
    __shared__ float s_Cf[KD], s_Hs[KD], s_Hv[KD], s_Ff[KD];
    // product form of the (dF/dC)^T pass: its per-codeword operands (c_j - mu, -s^2 |c_j - mu|^2, mu, h_j . (F*_j - mu) / tau),
    // formed by wavefront 0 -- the first three once per launch, the last whenever h changes -- from k d = 32 on (below,
    // every lane forms them itself at the start of its pass)
    constexpr bool BTAB = SmallItem<K, D, DIST, PASS_B2>::B2_DOT && !GLOBALW && KD >= 32;
    __shared__ float s_tabB[BTAB ? KD + K + D + K : 1];
    __shared__ int s_done, s_iters, s_conv, s_attempt, s_grow, s_halv, s_bad, s_restart;
    __shared__ double s_alpha, s_prev, s_vnorm, s_res;
    // minimal-residual solve (BWD_GMRES): offered to teams in which every workgroup receives the totals; its state lies
    // in the dynamic LDS at pa.gm_off (behind the tiles), only in launches of that mode
    extern __shared__ double s_dyn_d[];
    GmView<KD> gm;
    gm.bind(reinterpret_cast<char*>(s_dyn_d) + pa.gm_off, gm_basis_length(pa.gm_basis, KD));

    const int tid = threadIdx.x, wg = pa.wg;
    const int64_t base = (int64_t)wg * pa.per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < pa.per) ? (int)(a.m - base) : pa.per;
    const float* s_w = GLOBALW ? a.W : s_tile;
    const float* s_gt = GLOBALW ? a.G : s_tile + (size_t)pa.per * D;
    tree_announce(pa);
    if (!GLOBALW) {
        load_tile<PT>(s_tile, a.W + base * D, cnt * D);
        load_tile<PT>(s_tile + (size_t)pa.per * D, a.G + base * D, cnt * D);
    }
    if (tid < KD) {
        s_Cf[tid] = a.Cf[tid];
        s_Ff[tid] = a.Ff[tid];
        s_Hs[tid] = 0.f;
        s_Hv[tid] = 0.f;
    }
    float r_fm = 0.f;  // lane j d + r < k d of wavefront 0: F*_jr - mu_r
    if constexpr (BTAB) {
        if (tid < 64) {
            const float mu = fwd_dot_tables<K, D>(tid < KD ? a.Cf[tid] : 0.f, -a.nscale, s_tabB, 1.f);
            if (tid < KD) r_fm = a.Ff[tid] - mu;
        }
    }
    // every change of h/tau goes through here (lanes < k d of wavefront 0, all of them together)
    auto set_h = [&](float h) {
        s_Hs[tid] = h;
        if constexpr (BTAB) bwd_dot_hf<K, D>(h * r_fm, s_tabB);
    };
    if (tid < K) {
        const double n = a.nd[tid];
        s_rn[tid] = (n > 0.0) ? (double)a.inv_tau / n : 0.0;  // zero for an empty cluster
    }
    const int mode = pa.mode;
    const double tol = pa.tol;
    const int max_iter = pa.max_iter;
    if (tid == 0) {
        xs.abort = 0;
        s_done = (mode == BWD_JFB || mode == BWD_DENSE) ? 1 : 0;
        s_iters = 0;
        s_conv = (mode == BWD_JFB || mode == BWD_DENSE) ? 1 : 0;
        s_attempt = 0;
        s_grow = 0;
        s_halv = 0;
        s_bad = 0;
        s_restart = 0;
        s_alpha = pa.alpha;
        s_prev = __builtin_inf();
        s_vnorm = 0.0;
        s_res = 0.0;
    }
    __syncthreads();
    // (the explicit-Jacobian mode keeps the plain exchange: its one reduction is solved by workgroup 0)
    const bool tree = pa.tree && mode != BWD_DENSE;
    if (pa.tree && !tree_handshake(pa, xs)) return;
    unsigned int seq = pa.seq_base;

    float accr[SmallItem<K, D, DIST, PASS_B2>::NREG];            // (the (dF/dC)^T pass may keep more sums in registers than it publishes)
    float(&acc)[KD] = reinterpret_cast<float(&)[KD]>(accr);
    bool dense_done = false;
    if constexpr (HAS_DENSE) {
        if (mode == BWD_DENSE) {
            // one pass accumulates v and the sums T, U of dF/dC* (layout as in the stream path's tail_bj); workgroup 0
            // adds them over the team, solves (I - dF/dC*)^T g = v by Gauss-Jordan elimination and broadcasts h/tau
            float accj[NBJ];
            any_tile_pass<K, D, DIST, PASS_BJ, SHARED, GLOBALW>(a, pa, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, accj);
            ++seq;
            publish_partials<NBJ>(pa, seq, accj, xs);
            if (wg == 0) {
                __shared__ double s_tj[NBJ];
                __shared__ double s_M[KD * (KD + 1)];
                for (int first = 0; first < NBJ; first += 4) {
                    if (!reduce_slice<NBJ, 4>(pa, seq, first, xs)) return;
                    if (tid < 4) s_tj[first + tid] = xs.tot[tid];
                    __syncthreads();
                }
                if (tid == 0) {
                    constexpr int n = KD, n1 = KD + 1;
                    const double* T = s_tj;
                    const double* U = s_tj + n * n;
                    const double* V = s_tj + n * n + n * D;
                    for (int row = 0; row < n; ++row) {
                        const int l = row / D, sidx = row - l * D;
                        for (int col = 0; col < n; ++col) {
                            const int j = col / D;
                            const double J = ((l == j ? U[col * D + sidx] : 0.0) - T[col * n + row]) * s_rn[j];
                            s_M[row * n1 + col] = (row == col ? 1.0 : 0.0) - J;
                        }
                        s_M[row * n1 + n] = V[row];
                    }
                    bool sing = false;
                    for (int p = 0; p < n; ++p) {
                        int best = p;
                        double bv = fabs(s_M[p * n1 + p]);
                        for (int i = p + 1; i < n; ++i)
                            if (fabs(s_M[i * n1 + p]) > bv) {
                                bv = fabs(s_M[i * n1 + p]);
                                best = i;
                            }
                        if (!(bv > 1e-300) || !(bv <= 1.7e308)) sing = true;
                        if (best != p)
                            for (int j = 0; j < n1; ++j) {
                                const double x = s_M[p * n1 + j];
                                s_M[p * n1 + j] = s_M[best * n1 + j];
                                s_M[best * n1 + j] = x;
                            }
                        const double pp = s_M[p * n1 + p];
                        for (int i = 0; i < n; ++i) {
                            if (i == p) continue;
                            const double f = s_M[i * n1 + p] / pp;
                            for (int j = p; j < n1; ++j) s_M[i * n1 + j] -= f * s_M[p * n1 + j];
                        }
                    }
                    double v2 = 0.0;
                    for (int idx = 0; idx < n; ++idx) {
                        const double g = s_M[idx * n1 + n] / s_M[idx * n1 + idx];
                        if (!(fabs(g) <= 1.7e308)) sing = true;
                        s_g[idx] = g;
                        s_v[idx] = V[idx];
                        v2 += V[idx] * V[idx];
                        st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + idx], pack_f(seq, (float)(g * s_rn[idx / D])));
                    }
                    // a singular or non-finite system travels as a NaN norm: every workgroup then reports it
                    if (sing) v2 = __builtin_nan("");
                    for (int r = 0; r < R; ++r)
                        st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + KD + r], pack_f(seq, r == 0 ? (float)v2 : 0.f));
                }
            }
            dense_done = true;
        }
    }
    if (!dense_done) {
    // B1: v = dL/dC* with W fixed; the solve starts at g = v
    any_tile_pass<K, D, DIST, PASS_B1, SHARED, GLOBALW>(a, pa, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, acc);
    ++seq;
    publish_partials<KD>(pa, seq, acc, xs);
    if (tree) {
        // every workgroup holds the whole of v and starts the solve at g = v itself
        if (!tree_totals<KD>(pa, seq, xs)) return;
        if (tid < 64) {
            double v2 = 0.0;
            if (tid < KD) {
                const double v = xs.totd[tid];
                s_v[tid] = v;
                s_g[tid] = v;
                v2 = v * v;
                xs.bc[tid] = __float_as_uint((float)(v * s_rn[tid / D]));
            }
            v2 = first_lanes_sum_d_dpp<KD>(v2);
            if (tid < R) xs.bc[KD + tid] = (tid == 0) ? __float_as_uint((float)v2) : 0u;
        }
        __syncthreads();
    } else {
    for (int r = wg; r < R; r += pa.G) {
        if (!reduce_slice<KD, WPR>(pa, seq, r * WPR, xs)) return;
        if (tid < 64) {
            double v2 = 0.0;
            if (tid < WPR) {
                const int idx = r * WPR + tid;
                const double v = xs.tot[tid];
                s_v[idx] = v;
                s_g[idx] = v;
                v2 = v * v;
                const float h = (float)(v * s_rn[idx / D]);
                st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + idx], pack_f(seq, h));
                xs.bc[idx] = __float_as_uint(h);
            }
            v2 = first_lanes_sum_d_dpp<WPR>(v2);
            if (tid == 0) {
                st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + KD + r], pack_f(seq, (float)v2));
                xs.bc[KD + r] = __float_as_uint((float)v2);
            }
        }
    }
    }
    }
    if (!(tree && !dense_done) && !gather_bcast<KD, WPR, KD>(pa, seq, NB, !dense_done, xs)) return;
    if (tid < KD) {
        set_h(__uint_as_float(xs.bc[tid]));
        s_Hv[tid] = __uint_as_float(xs.bc[tid]);
    }
    if (tid == 0) {
        double v2 = 0.0;
        for (int r = 0; r < R; ++r) v2 += (double)__uint_as_float(xs.bc[KD + r]);
        s_vnorm = v2;  // squared norms throughout the solve; roots are taken when it is over
        if (!(v2 <= 1.7e308)) {
            s_bad = 1;
            s_done = 1;
        }
    }
    __syncthreads();
    {
        if (mode == BWD_GMRES && !s_done) {
            // from g = 0: the first residual is v itself, the first basis vector v / ||v||  (every workgroup holds v)
            if (tid < 64) {
                double v2 = 0.0;
                if (tid < KD) v2 = s_v[tid] * s_v[tid];
                v2 = first_lanes_sum_d_dpp<KD>(v2);
                v2 = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(v2)),
                                      __builtin_amdgcn_readfirstlane(__double2loint(v2)));
                const double vn = sqrt(v2), inv = v2 > 0.0 ? 1.0 / vn : 0.0;
                if (tid < KD) {
                    const double q = s_v[tid] * inv;
                    gm.Q[tid] = q;
                    s_g[tid] = 0.0;
                    set_h((float)(q * s_rn[tid / D]));
                }
                if (tid == 0) {
                    s_vnorm = v2;  // (the float64 norm of the float64 v, not the sum of float32 parts)
                    gm.ctl[0] = 0;
                    gm.ctl[1] = 0;
                    gm.ctl[2] = 0;
                    gm.beta[0] = vn;
                    gm.sv[0] = vn;
                    if (v2 == 0.0) {  // v = 0: g = 0 is the solution
                        s_conv = 1;
                        s_done = 1;
                    }
                }
            }
            __syncthreads();
        }
    }

    // Where every workgroup receives the totals (a team of one, the two-level exchange) wavefront 0 keeps the state of
    // the averaged iteration in registers -- its own element of g, v and 1/(tau n), the damping factor, the counters of
    // the restart rule -- and every lane takes the same decision from the same step norm: between the arrival of the
    // totals and the next pass there is then one barrier and no read of that state from LDS.
    double r_g = 0.0, r_v = 0.0, r_rn = 0.0, r_alpha = pa.alpha, r_prev = __builtin_inf();
    const double vnorm2 = s_vnorm;
    int r_grow = 0, r_attempt = 0, r_halv = 0, r_iters = 0;
    if (tid < KD) {
        r_g = s_g[tid];
        r_v = s_v[tid];
        r_rn = s_rn[tid / D];
    }
    while (!s_done) {
        IDKM_STAMP(0);
        any_tile_pass<K, D, DIST, PASS_B2, SHARED, GLOBALW>(a, pa, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, accr, BTAB ? s_tabB : nullptr);
        IDKM_STAMP(1);
        ++seq;
        publish_partials<KD>(pa, seq, acc, xs);
        IDKM_STAMP(2);
        {
            if (mode == BWD_GMRES) {
                // (offered only where every workgroup receives the totals: a team of one, or the two-level exchange)
                if (tree) {
                    if (!tree_totals<KD>(pa, seq, xs)) return;
                } else {
                    __syncthreads();
                }
                if (tid < 64) {
                    double hn;
                    const double vn = fast_sqrt_d(s_vnorm);
                    int over;
                    if (tree)
                        over = gmres_step<KD>(gm, [&](int i) { return xs.totd[i]; }, s_v, s_g, tol, vn, max_iter, s_iters,
                                              s_conv, s_bad, s_res, hn);
                    else
                        over = gmres_step<KD>(gm, [&](int i) { return (double)xs.own[i]; }, s_v, s_g, tol, vn, max_iter,
                                              s_iters, s_conv, s_bad, s_res, hn);
                    if (tid < KD) set_h((float)(hn * s_rn[tid / D]));
                    if (tid == 0 && over) s_done = 1;
                }
                __syncthreads();
                continue;
            }
        }
        if (pa.G == 1 || tree) {
            // a team of one has no exchange: its partial sums (xs.own) are the totals; with the two-level exchange
            // every workgroup receives the totals (xs.totd).  Either way the whole of g is updated here
            bool wave0_abort = false;
            double u_reg = 0.0;   // (total of this lane's component where hop 2 leaves the totals in registers)
            bool in_regs = false;
            if (tree) {
                if constexpr (KD <= WAVE_WORDS_MAX) {
                    // (hop 2 inside wavefront 0, no barrier and no LDS round trip before the update)
                    if (wg < DIES && !tree8_die_totals(pa, seq, xs)) return;
                    if (tid < 64) {
                        double total;
                        wave0_abort = !tree8_grid_totals_regs(pa, seq, xs, total);
                        u_reg = tree8_total_of(total, tid < KD ? tid : 0);
                        in_regs = true;
                    }
                } else {
                    if (!tree_totals<KD>(pa, seq, xs)) return;
                }
            } else {
                __syncthreads();
            }
            IDKM_STAMP(4);
            if (tid < 64 && !wave0_abort) {
                double d2 = 0.0, gn = 0.0;
                if (tid < KD) {
                    const double u = in_regs ? u_reg : (tree ? xs.totd[tid] : (double)xs.own[tid]);
                    gn = r_alpha * (r_v + u) + (1.0 - r_alpha) * r_g;
                    const double df = gn - r_g;
                    d2 = df * df;
                }
                d2 = first_lanes_sum_d_dpp<KD>(d2);
                // the squared step norm as every lane sees it (rounded to float32 like the word the plain exchange
                // broadcasts, so that all forms of the exchange take the same decisions)
                const double dn = (double)__uint_as_float((unsigned int)__builtin_amdgcn_readfirstlane((int)__float_as_uint((float)d2)));
                bool restart = false, done = false, conv = false, diverged = false, bad = false;
                int grow = r_grow;
                const int attempt = r_attempt + 1;
                if (!(dn <= 1.7e308)) {
                    diverged = true;
                } else if (dn <= tol * tol * vnorm2) {
                    conv = true;
                    done = true;
                } else {
                    grow = (dn > r_prev) ? grow + 1 : 0;
                    if (grow >= 5) diverged = true;
                }
                if (!done && !diverged && attempt >= max_iter) done = true;
                if (diverged) {
                    if (r_halv < 6) {
                        restart = true;
                    } else {
                        done = true;
                        if (!(dn <= 1.7e308)) bad = true;  // every damping factor tried ended in a non-finite step
                    }
                }
                r_iters += 1;
                if (restart) {
                    // back to g = v with the halved alpha
                    r_alpha *= 0.5;
                    r_halv += 1;
                    r_attempt = 0;
                    r_grow = 0;
                    r_prev = __builtin_inf();
                    r_g = r_v;
                } else {
                    r_attempt = attempt;
                    r_grow = grow;
                    if (!diverged && !conv) r_prev = dn;
                    r_g = gn;
                }
                if (tid < KD) {
                    s_g[tid] = r_g;
                    set_h(restart ? s_Hv[tid] : (float)(gn * r_rn));
                }
                if (tid == 0) {  // (stores only)
                    s_iters = r_iters;
                    s_res = dn;
                    s_alpha = r_alpha;
                    if (conv) s_conv = 1;
                    if (bad) s_bad = 1;
                    if (done) s_done = 1;
                }
            }
            __syncthreads();
            if (xs.abort) return;
            continue;
        }
        const double alpha = s_alpha;
        {
        for (int r = wg; r < R; r += pa.G) {
            if (!reduce_slice<KD, WPR>(pa, seq, r * WPR, xs)) return;
            if (tid < 64) {
                double d2 = 0.0;
                if (tid < WPR) {
                    const int idx = r * WPR + tid;
                    const double g = s_g[idx];
                    const double gn = alpha * (s_v[idx] + xs.tot[tid]) + (1.0 - alpha) * g;
                    const double df = gn - g;
                    d2 = df * df;
                    s_g[idx] = gn;
                    const float h = (float)(gn * s_rn[idx / D]);
                    st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + idx], pack_f(seq, h));
                    xs.bc[idx] = __float_as_uint(h);
                }
                d2 = first_lanes_sum_d_dpp<WPR>(d2);
                if (tid == 0) {
                    st_word(&pa.buf2[(size_t)(seq & 1u) * XBCAST + KD + r], pack_f(seq, (float)d2));
                    xs.bc[KD + r] = __float_as_uint((float)d2);
                }
            }
            IDKM_STAMP(3);
        }
        if (!gather_bcast<KD, WPR, KD>(pa, seq, NB, true, xs)) return;
        }
        IDKM_STAMP(4);
        if (tid == 0) {
            // the same decision in every workgroup (same words, same order)
            double d2 = 0.0;
            for (int r = 0; r < R; ++r) d2 += (double)__uint_as_float(xs.bc[KD + r]);
            const double dn = d2;  // squared step norm: every comparison below is between squares
            bool restart = false, done = false, conv = false, diverged = false;
            int grow = s_grow;
            const int attempt = s_attempt + 1;
            if (!(dn <= 1.7e308)) {
                diverged = true;
            } else if (dn <= tol * tol * s_vnorm) {
                conv = true;
                done = true;
            } else {
                grow = (dn > s_prev) ? grow + 1 : 0;
                if (grow >= 5) diverged = true;
            }
            if (!done && !diverged && attempt >= max_iter) done = true;
            if (diverged) {
                if (s_halv < 6) {
                    restart = true;
                } else {
                    done = true;
                    if (!(dn <= 1.7e308)) s_bad = 1;  // every damping factor tried ended in a non-finite step
                }
            }
            IDKM_STAMP(5);
            s_iters += 1;
            s_res = dn;
            if (conv) s_conv = 1;
            if (restart) {
                s_alpha = alpha * 0.5;
                s_halv += 1;
                s_attempt = 0;
                s_grow = 0;
                s_prev = __builtin_inf();
            } else {
                s_attempt = attempt;
                s_grow = grow;
                if (!diverged && !conv) s_prev = dn;
            }
            s_restart = restart ? 1 : 0;
            if (done) s_done = 1;
        }
        __syncthreads();
        if (s_restart) {
            // back to g = v with the halved alpha: every workgroup kept h(v)/tau, reducers reset their slice
            if (tid < KD) {
                set_h(s_Hv[tid]);
                s_g[tid] = s_v[tid];
            }
        } else if (tid < KD) {
            set_h(__uint_as_float(xs.bc[tid]));
        }
        __syncthreads();
    }

    // B3: dW = direct + (dF/dW)^T g
    any_tile_pass<K, D, DIST, PASS_B3, SHARED, GLOBALW>(a, pa, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, reinterpret_cast<float(&)[1]>(acc[0]));
    if (dense_done || tree) {
        if (wg == 0 && tid < KD) {
            a.gd[tid] = s_g[tid];
            a.vd[tid] = s_v[tid];
        }
    } else {
        for (int r = wg; r < R; r += pa.G) {
            if (tid < WPR) {
                const int idx = r * WPR + tid;
                a.gd[idx] = s_g[idx];
                a.vd[idx] = s_v[idx];
            }
        }
    }
    if (wg == 0 && tid < KD) a.Hs[tid] = s_Hs[tid];
    if (wg == pa.G - 1 && tid == 0) {
        PResult* o = pa.out;
        o->iters = s_iters;
        o->converged = s_conv;
        o->residual = sqrt(s_res);
        o->alpha = s_alpha;
        o->vnorm = sqrt(s_vnorm);
        o->halvings = s_halv;
        o->nonfinite = s_bad;
        o->done = pa.seq_base + 1u;
    }
}

// One team per launch: the grid is the team.
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_fwd(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_fwd_body<K, D, DIST, false>(a, pa);
}
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_bwd(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_bwd_body<K, D, DIST, false>(a, pa);
}

// The same for a layer larger than the chip's LDS (W is read from memory in every pass; no dynamic LDS).
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_fwd_global(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_fwd_body<K, D, DIST, false, true>(a, pa);
}
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_bwd_global(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_bwd_body<K, D, DIST, false, true>(a, pa);
}

// Several independent problems of one shape (the layers of Alg. 2's loops) in one launch: item_of_wg maps a
// workgroup to its problem; every team runs its own solve and leaves when that solve is over.
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_fwd_batch(const BatchItem* items, const unsigned short* item_of_wg) {
    const BatchItem& it = items[item_of_wg[blockIdx.x]];
    const Args a = it.a;
    PArgs pa = it.p;
    pa.wg = (int)blockIdx.x - it.wg_begin;
    pa.G = it.wg_count;
    persist_fwd_body<K, D, DIST, true>(a, pa);
}
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_bwd_batch(const BatchItem* items, const unsigned short* item_of_wg) {
    const BatchItem& it = items[item_of_wg[blockIdx.x]];
    const Args a = it.a;
    PArgs pa = it.p;
    pa.wg = (int)blockIdx.x - it.wg_begin;
    pa.G = it.wg_count;
    persist_bwd_body<K, D, DIST, true>(a, pa);
}

}  // namespace idkm
