// Fused single-sequence decode step (Sec. 3.3 "Decoding Stage", Sec. 3.4 two-step decoding).
//
// One launch streams, exactly once, the weights the step needs: gate+up rows of the retained and candidate
// channels and down columns of the retained and selected channels, each channel's block w[j] = [gate|up|down]
// being contiguous in memory.
//
// Work unit: a "round" handled by one whole workgroup.  The workgroup's threads split the d columns (thread t owns
// 16-byte vector column t), so a channel's gate, up and down rows are each read by one coalesced sweep of the
// workgroup, x and the partial y live in registers (no LDS staging, no reduction of y across waves), and the only
// exchange is the per-row gate/up dot product: wave partials go through LDS, one barrier per round.  The next
// round's rows are requested as soon as the current round's data has been consumed, so the reduction and the
// barrier overlap the memory latency.
//
// A round carries kRB retained channels (gate, up and down rows: h_j = silu(g_j) u_j, then y += h_j * down_j) and
// kXL extra rows that ride along:
//   - first the workgroup's share of the candidate channels (gate+up only): h_j and the step score
//     I_j(t) = n_j |h_j| (Eq. 3 with one token) are published to global memory with write-through stores.  The
//     selection waits for every workgroup's candidates, so they go first: four per round (the retained channels'
//     gate and up buffers take two of them) while three or more are left, the last one or two next to retained
//     channels;
//   - later, once the selection is known, the down rows of those of its own candidates that were selected.
// Candidates are dealt round-robin to all workgroups, retained rounds round-robin to the workers: the schedule,
// and with it the summation order of y, is fixed (bit-reproducible output).  (Letting workers draw part of their
// rounds from shared ticket counters at run time was tried: the requests have to be issued several rounds ahead to
// keep their latency out of the stream, and with that much claimed-ahead work the finishing times did not even
// out; it measured 3 % slower.)
//
//   select   workgroup 0 owns no retained rows.  It collects every candidate's h (bounded wait; nobody waits for
//            anything before that point), forms the step scores, runs the top-k selection and hands every workgroup
//            one word: one bit per candidate slot of that workgroup that was selected.  Mask and active list for the
//            caller are written afterwards.
//   poll     a worker looks at its word once per round without ever stalling on it (thread 0 passes the value
//            loaded in the previous round to the others through LDS, at the round's barrier); if the word has not
//            arrived when the retained rounds are done the workgroup waits, bounded.
//   output   every workgroup leaves its partial y as one row; a second small kernel (decode_tail_kernel) sums the
//            rows in workgroup order and writes y.
//
// Hand-overs carry their own validity.  Everything one workgroup hands to another inside the launch (a candidate's
// h, a selection word) is a 64-bit word {value, epoch} written with one write-through store and read
// with one device-coherent load; the epoch is a device-resident counter that the last workgroup of a launch
// increments.  A reader that finds another epoch sees "not there yet" and looks again.  There are no counters or
// flags to clear or re-arm, words of an earlier step (or of a step that gave up) can never be taken for valid, and
// a captured launch can be replayed.
//
// Waiting is safe because the launch is sized to be co-resident (host checks the occupancy) and every wait is
// bounded; nothing spins without an exit.  A wait that expires raises the sticky error flag (the step's results
// are then invalid) and changes nothing else: every workgroup still reaches the end, and the next launch starts
// from a new epoch.
#include <limits.h>
#include <type_traits>
#include <stdlib.h>

#include "pop_select_dev.h"
#include "pop_vec.h"

namespace pop {

constexpr int kRB = 2;           // retained channels per round
constexpr int kXL = 4;           // extra rows per round: 2 candidates x (gate, up), or 4 selected down rows
constexpr int kMaxStatic = 64;   // statically dealt rounds per workgroup (staged in LDS)
constexpr int kKeep = 64;        // rounds whose hidden activations are staged in LDS between flushes
constexpr int kMaxASlots = 30;   // candidate slots per workgroup: they must fit the selection word next to the valid bit

// Optional per-workgroup timestamps (100 MHz wall clock), compiled in only for profiling builds.
#ifdef POP_TRACE
#define POP_STAMP(slot)                                                                 \
    do {                                                                                \
        if (p.trace && threadIdx.x == 0) p.trace[(size_t)blockIdx.x * 8 + (slot)] = wall_clock64(); \
    } while (0)
#else
#define POP_STAMP(slot) \
    do {                \
    } while (0)
#endif

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <class V, int PER>
struct RoundBuf {
    typename V::vec_t g[kRB][PER], u[kRB][PER], dn[kRB][PER], xl[kXL][PER];
};

// What a round holds; the same in every thread of the workgroup (kept in scalar registers).
struct RoundDesc {
    int jb[kRB];    // retained channels, -1 = empty slot
    int xrow[kXL];  // the extra rows, as row numbers of w viewed as [3 m][d] (-1 = none): gate and up rows of two
                    // candidates (xkind 1) or down rows of up to four selected candidates (xkind 2)
    int xmeta;      // bits 0-1 xkind, bit 2 "this round completes the workgroup's candidates",
                    // bits 8+5a .. 12+5a the candidate slot in this workgroup of extra item a
    int bmeta;      // 0: jb are retained channels.  Bit 0 set: a round of candidates only - jb are two more of the
                    // workgroup's candidates (gate and up rows, no down row), bits 8+8t .. 15+8t their slots
    uint32_t boff[kRB], xoff[kXL];  // where those rows start in w, in 16-byte vectors (0 for an empty slot):
                                    // worked out with the descriptor, a round before the rows are requested
    bool work;      // the round holds anything at all
    __device__ __forceinline__ int xkind() const { return xmeta & 3; }
    __device__ __forceinline__ bool last_a() const { return (xmeta & 4) != 0; }
    __device__ __forceinline__ int xslot(int a) const { return (xmeta >> (8 + 5 * a)) & 31; }
    __device__ __forceinline__ bool bcand() const { return (bmeta & 1) != 0; }
    __device__ __forceinline__ int bslot(int t) const { return (bmeta >> (8 + 8 * t)) & 255; }
};

// Requests the rows of one round: the extra rows first (only in rounds that have any: a request for a dummy
// vector still occupies the cache's return path for a full wave), then the retained channels' rows, always and in
// the same order, with no branch around them (an empty slot or an out-of-range column reads the first 16 bytes of
// w): the compiler then knows how many requests are younger than the rows it needs and waits for no others.
// The down rows come last: they are needed last.  Addresses are w + 16 * (32-bit vector index).
template <class V, int PER>
__device__ __forceinline__ void load_round(RoundBuf<V, PER> &rb, const RoundDesc &ds,
                                           const typename V::vec_t *__restrict__ w, int nvec, const int (&col)[PER],
                                           const bool (&ok)[PER])
{
    if (ds.xmeta != 0) {
#pragma unroll
        for (int a = 0; a < kXL; ++a)
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const uint32_t idx = (ok[q] && ds.xrow[a] >= 0) ? ds.xoff[a] + (uint32_t)col[q] : 0u;
                rb.xl[a][q] = w[idx];
            }
    }
    uint32_t idx[kRB][PER];
#pragma unroll
    for (int t = 0; t < kRB; ++t)
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const bool ld = ok[q] && ds.jb[t] >= 0;
            idx[t][q] = ld ? ds.boff[t] + (uint32_t)col[q] : 0u;
            rb.g[t][q] = w[idx[t][q]];
            rb.u[t][q] = w[ld ? idx[t][q] + (uint32_t)nvec : 0u];
        }
#pragma unroll
    for (int t = 0; t < kRB; ++t)
#pragma unroll
        for (int q = 0; q < PER; ++q)
            rb.dn[t][q] = w[(ok[q] && ds.jb[t] >= 0 && !ds.bcand()) ? idx[t][q] + 2u * (uint32_t)nvec : 0u];
}

// Sum over the 16 lanes of each DPP row, result in every lane of the row (4 cross-lane adds, no LDS).
__device__ __forceinline__ float dpp_row_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));   // quad_perm 1,0,3,2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));   // quad_perm 2,3,0,1
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));  // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true));  // row_mirror
    return v;
}

__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__device__ __forceinline__ float wave_total(float v)
{
    const float r = dpp_row_sum(v);
    return (lane_value(r, 0) + lane_value(r, 16)) + (lane_value(r, 32) + lane_value(r, 48));
}

// 16-byte write-through store (device scope), p 16-byte aligned.  Not tracked by the compiler's wait counting:
// follow with an explicit wait before relying on it.
__device__ __forceinline__ void coherent_store4(float *p, float4 v)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 t = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(t) : "memory");
}

constexpr int kSelStride = 16;       // 64-bit words between the selection words of two workgroups (128 bytes)
constexpr int kBitsValid = 1 << 31;  // set, next to the slot bits, in the copy of a selection word that thread 0
                                     // hands to its workgroup once the word carries the step's epoch

__device__ __forceinline__ unsigned long long tagged(uint32_t value, int epoch)
{
    return ((unsigned long long)(uint32_t)epoch << 32) | value;
}
__device__ __forceinline__ void coherent_store(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// sum over the vector's elements of (g_e^2 + u_e^2) * x_e^2, added to acc: a candidate's importance under the
// input-side reading of Eq. 1-2 with one token (all terms are positive: no cancellation)
__device__ __forceinline__ float sq_dot(const uint4 &g, const uint4 &u, const uint4 &x, float acc)
{
    const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w}, xw[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float xl = bf16_lo(xw[e]), xh = bf16_hi(xw[e]);
        const float gl = bf16_lo(gw[e]), gh = bf16_hi(gw[e]), ul = bf16_lo(uw[e]), uh = bf16_hi(uw[e]);
        acc = fmaf(fmaf(gl, gl, ul * ul), xl * xl, acc);
        acc = fmaf(fmaf(gh, gh, uh * uh), xh * xh, acc);
    }
    return acc;
}
__device__ __forceinline__ double sq_dot(const float4 &g, const float4 &u, const float4 &x, double acc)
{
    const float gv[4] = {g.x, g.y, g.z, g.w}, uv[4] = {u.x, u.y, u.z, u.w}, xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const double gg = (double)gv[e], uu = (double)uv[e], xx = (double)xs[e];
        acc = fma(fma(gg, gg, uu * uu), xx * xx, acc);
    }
    return acc;
}

template <class V, int PER, int MAXB>
__global__ __launch_bounds__(MAXB) void decode_fused_kernel(FusedParams p)
{
    typedef typename V::vec_t vec_t;
    typedef typename V::acc_t acc_t;
    constexpr int E = V::kElems;
    __shared__ SelShared sh;
    __shared__ int s_flag;
    __shared__ int mb_bits[2];  // thread 0 -> everyone, handed over at the round's barrier
    // wave partials of the dot products, summed in double: [parity][group: retained, extras][value][wave][row of 16 lanes]
    // (third group: the candidates' input-side importance sums, when that reading is on)
    __shared__ __attribute__((aligned(32))) double part[2][3][4][kSelMaxWaves][4];
    __shared__ int j_s[(kMaxStatic + 1) * kRB];                     // statically dealt retained channels
    __shared__ int j_a[32];                                         // this workgroup's candidates, by slot
    __shared__ float h_a[32];                                       // their hidden activations
    __shared__ float q_a[32];                                       // their step scores (input-side reading only)
    __shared__ int j_st[kKeep * kRB];                               // retained channels processed since the last flush
    __shared__ float h_st[kKeep * kRB];                             // and their hidden activations
    __shared__ int wg_bits[1024];                                   // selector only: selected candidate slots per workgroup

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int b = blockIdx.x, n_wg = gridDim.x, n_workers = n_wg - 1, wb = b - 1;
    const int nvec = p.nvec;
    const vec_t *w = reinterpret_cast<const vec_t *>(p.w);
    unsigned long long *const my_word = p.selw + (size_t)b * kSelStride;
    const int epoch = coherent_load(&p.ctr[0]);  // the tag of everything handed over in this step
    const int limit = p.spin_limit;
    const bool input_side = p.input_side != 0;

    POP_STAMP(0);
    int col[PER];
    bool ok[PER];
    vec_t xv[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        col[q] = tid + q * blockDim.x;
        ok[q] = col[q] < nvec;
        xv[q] = ok[q] ? reinterpret_cast<const vec_t *>(p.x)[col[q]] : V::zero();
    }
    for (int i = tid; i < 2 * 3 * 4 * kSelMaxWaves * 4; i += blockDim.x) (&part[0][0][0][0][0])[i] = 0;

    // ---- this workgroup's share
    // candidates: slot s of workgroup b is candidate s * n_wg + b
    const int n_aslots = b < p.n_cand ? (p.n_cand - b + n_wg - 1) / n_wg : 0;
    // retained: round i of worker wb covers ret_idx[(i * n_workers + wb) * kRB ..]
    const int n_static = wb >= 0 ? p.n_static : 0;
    const int static_end = p.n_ret;
    if (tid < 32) j_a[tid] = tid < n_aslots ? p.cand_idx[tid * n_wg + b] : -1;
    for (int e = tid; e < (n_static + 1) * kRB; e += blockDim.x) {
        const int r = ((e / kRB) * n_workers + wb) * kRB + e % kRB;
        j_s[e] = (e / kRB < n_static && r < static_end) ? p.ret_idx[r] : -1;
    }
    if (tid < 2) mb_bits[tid] = 0;
    __syncthreads();

    // partial y of the retained channels, and of the selected candidates: kept apart and added at the end, so that
    // the summation order does not depend on the round in which the selection happened to arrive
    float acc[PER][8], acc_sel[PER][8];
#pragma unroll
    for (int q = 0; q < PER; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = acc_sel[q][e] = 0.f;

    // ---- round state, identical in every thread
    int ia = 0;                 // next candidate slot to evaluate
    int rem_d = 0;              // selected slots whose down rows are still to be added (valid once bits_known)
    bool bits_known = false;    // the selection word of this step has been seen
    int n_st = 0;               // rounds staged in j_st / h_st
    // thread 0 only: the selection word as polled in the previous round
    unsigned long long poll_ret = 0;

    // Descriptor of the next round.  Called once per round, in order.  While the workgroup has three or more
    // candidates left, a round holds candidates only, four at a time (two in the extra rows, two in the retained
    // channels' gate and up buffers): the candidates' results are what the selection waits for, so they go out
    // first, in rounds that still carry 64 KB.  The last one or two ride along with retained rounds.
    int ir = 0;  // next retained round of this worker
    auto make_desc = [&](RoundDesc &ds) {
        bool work = false;
#pragma unroll
        for (int t = 0; t < kRB; ++t) ds.jb[t] = -1;
        ds.bmeta = 0;
        ds.xmeta = 0;
#pragma unroll
        for (int a = 0; a < kXL; ++a) ds.xrow[a] = -1;
        const bool cand_round = n_aslots - ia >= 3;
        if (!cand_round && ir < n_static) {
#pragma unroll
            for (int t = 0; t < kRB; ++t) ds.jb[t] = uniform(j_s[ir * kRB + t]);
            work = ds.jb[0] >= 0;
            ++ir;
        }
        if (ia < n_aslots) {
            ds.xmeta = 1;
#pragma unroll
            for (int a = 0; a < 2; ++a)
                if (ia + a < n_aslots) {
                    const int j = uniform(j_a[ia + a]);
                    ds.xmeta |= (ia + a) << (8 + 5 * a);
                    ds.xrow[2 * a] = j * 3;
                    ds.xrow[2 * a + 1] = j * 3 + 1;
                }
            ia += 2;
            if (cand_round) {
                ds.bmeta = 1;
#pragma unroll
                for (int t = 0; t < kRB; ++t)
                    if (ia + t < n_aslots) {
                        ds.jb[t] = uniform(j_a[ia + t]);
                        ds.bmeta |= (ia + t) << (8 + 8 * t);
                    }
                ia += 2;
            }
            if (ia >= n_aslots) ds.xmeta |= 4;
            work = true;
        } else if (bits_known && rem_d && work) {
            // selected rows ride along with retained rounds only: on their own they would cost a full trip to
            // memory per round, while the drain after the loop requests them all at once
            ds.xmeta = 2;
#pragma unroll
            for (int a = 0; a < kXL; ++a)
                if (rem_d) {
                    const int sl = __builtin_ctz(rem_d);
                    rem_d &= rem_d - 1;
                    ds.xmeta |= sl << (8 + 5 * a);
                    ds.xrow[a] = uniform(j_a[sl]) * 3 + 2;
                }
            work = true;
        }
#pragma unroll
        for (int t = 0; t < kRB; ++t) ds.boff[t] = (uint32_t)max(ds.jb[t], 0) * 3u * (uint32_t)nvec;
#pragma unroll
        for (int a = 0; a < kXL; ++a) ds.xoff[a] = (uint32_t)max(ds.xrow[a], 0) * (uint32_t)nvec;
        ds.work = work;
    };

    // all threads write the staged hidden activations of the retained channels out (between barriers)
    auto flush_hidden = [&]() {
        __syncthreads();
        for (int e = tid; e < n_st * kRB; e += blockDim.x)
            if (j_st[e] >= 0) p.h[j_st[e]] = h_st[e];
        __syncthreads();
        n_st = 0;
    };

    // One round: reduce the rows in `cur` (round i, descriptor dc).  Right after their gate/up data has been
    // consumed the rows of round i + 1 are requested into `nxt` (descriptor dn1, prepared a round earlier, so that
    // nothing stands between the arrival of one round and the request for the next); the descriptor of round i + 2
    // is prepared into dn2 while that request is in flight.
    auto step = [&](RoundBuf<V, PER> &cur, const RoundDesc &dc, RoundBuf<V, PER> &nxt, const RoundDesc &dn1,
                    RoundDesc &dn2, int i, auto parity) {
        constexpr int par = decltype(parity)::value;  // i & 1
        const int xkind = dc.xkind();
        acc_t ag[kRB], au[kRB], ax[kXL];
#pragma unroll
        for (int t = 0; t < kRB; ++t) {
            ag[t] = 0;
            au[t] = 0;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                ag[t] = V::dot(cur.g[t][q], xv[q], ag[t]);
                au[t] = V::dot(cur.u[t][q], xv[q], au[t]);
            }
        }
        // The extra rows are multiplied in every round, needed or not (16 instructions): a register that is loaded
        // on some paths and read on others would count as "possibly still in flight" for the rest of the loop,
        // and the compiler would then wait for every outstanding request before reusing it.
#pragma unroll
        for (int a = 0; a < kXL; ++a) {
            ax[a] = 0;
#pragma unroll
            for (int q = 0; q < PER; ++q) ax[a] = V::dot(cur.xl[a][q], xv[q], ax[a]);
        }
        // input-side reading: a candidate's step score comes from the same two rows, sum (g^2 + u^2) x_t^2
        acc_t aq[4] = {0, 0, 0, 0};
        if (input_side && xkind == 1) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int q = 0; q < PER; ++q) aq[a] = sq_dot(cur.xl[2 * a][q], cur.xl[2 * a + 1][q], xv[q], aq[a]);
            if (dc.bcand()) {
#pragma unroll
                for (int t = 0; t < kRB; ++t)
#pragma unroll
                    for (int q = 0; q < PER; ++q) aq[2 + t] = sq_dot(cur.g[t][q], cur.u[t][q], xv[q], aq[2 + t]);
            }
        }
        asm volatile("" ::: "memory");  // everything below stays behind the uses of this round's gate/up rows
        if (tid == 0) {
            // The poll of the selection word that thread 0 issued in the previous round is older than this round's
            // rows, which have arrived: hand it to the others at this round's barrier.  Then poll again (another
            // epoch until the selector has written the word), ahead of the next round's requests.
            const bool here = (int)(poll_ret >> 32) == epoch;
            mb_bits[par] = here ? ((int)(uint32_t)poll_ret | kBitsValid) : 0;
#ifdef POP_TRACE
            if (here && p.trace && p.trace[(size_t)blockIdx.x * 8 + 5] == 0) POP_STAMP(5);
#endif
            poll_ret = coherent_load(my_word);
        }
        asm volatile("" ::: "memory");
        load_round<V, PER>(nxt, dn1, w, nvec, col, ok);  // an empty round requests the dummy vector only
        asm volatile("" ::: "memory");

        // wave partials -> LDS -> totals in every thread (one barrier)
        // (a thread's one or two vectors of products are summed in the row's accumulator type; across lanes and
        // waves the sums run in double, so the tree adds no float32 rounding at the magnitude of the full sum).  Each
        // group of four values goes through halving exchanges inside the 16-lane rows; the four row sums of each wave
        // meet the other waves' in LDS: one barrier per round
        static_assert(kRB == 2 && kXL == 4, "two groups of four values: gate/up of two retained channels, four extra rows");
        {
            const double a4[4] = {(double)ag[0], (double)au[0], (double)ag[1], (double)au[1]};
            const double z = butterfly4_row_sum(a4, lane);
            if (lane % 16 < 4) part[par][0][butterfly_value_id(lane)][wave][lane / 16] = z;
            if (xkind == 1) {
                const double x4[4] = {(double)ax[0], (double)ax[1], (double)ax[2], (double)ax[3]};
                const double zx = butterfly4_row_sum(x4, lane);
                if (lane % 16 < 4) part[par][1][butterfly_value_id(lane)][wave][lane / 16] = zx;
                if (input_side) {
                    const double q4[4] = {(double)aq[0], (double)aq[1], (double)aq[2], (double)aq[3]};
                    const double zq = butterfly4_row_sum(q4, lane);
                    if (lane % 16 < 4) part[par][2][butterfly_value_id(lane)][wave][lane / 16] = zq;
                }
            }
        }
        __syncthreads();
        // descriptor of round i + 2, with what thread 0 handed over at this barrier
        if (!bits_known) {
            const int v = uniform(mb_bits[par]);
            if (v & kBitsValid) {
                bits_known = true;
                rem_d = v & ~kBitsValid;
                POP_STAMP(7);
            }
        }
        make_desc(dn2);
        float hv[kRB], hx[2] = {0.f, 0.f}, sx[4] = {0.f, 0.f, 0.f, 0.f};
        {
            // lane l: value l / 16 of wave l % 16 (unused waves' slots stay zero): its four row sums, then a row sum
            // over the 16 lanes adds the waves in a fixed tree order
            const double4 q4 = *reinterpret_cast<const double4 *>(&part[par][0][lane / 16][lane % 16][0]);
            const double tot = dpp_row_sum((q4.x + q4.y) + (q4.z + q4.w));
#pragma unroll
            for (int t = 0; t < kRB; ++t)
                hv[t] = dc.jb[t] >= 0 ? silu_mul((float)lane_value(tot, 32 * t), (float)lane_value(tot, 32 * t + 16)) : 0.f;
            if (xkind == 1) {
                const double4 x4 = *reinterpret_cast<const double4 *>(&part[par][1][lane / 16][lane % 16][0]);
                const double tx = dpp_row_sum((x4.x + x4.y) + (x4.z + x4.w));
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    hx[a] = dc.xrow[2 * a] >= 0
                                ? silu_mul((float)lane_value(tx, 32 * a), (float)lane_value(tx, 32 * a + 16))
                                : 0.f;
                if (input_side) {
                    const double4 s4 = *reinterpret_cast<const double4 *>(&part[par][2][lane / 16][lane % 16][0]);
                    const double ts = dpp_row_sum((s4.x + s4.y) + (s4.z + s4.w));
#pragma unroll
                    for (int a = 0; a < 4; ++a) sx[a] = sqrtf((float)lane_value(ts, 16 * a));
                }
            }
        }
        const bool bcand = dc.bcand();
        if (tid == 0) {
            if (bcand) {
#pragma unroll
                for (int t = 0; t < kRB; ++t)
                    if (dc.jb[t] >= 0) {
                        h_a[dc.bslot(t)] = hv[t];
                        q_a[dc.bslot(t)] = sx[2 + t];
                    }
            } else if (dc.jb[0] >= 0) {
#pragma unroll
                for (int t = 0; t < kRB; ++t) {
                    j_st[n_st * kRB + t] = dc.jb[t];
                    h_st[n_st * kRB + t] = hv[t];
                }
            }
            if (xkind == 1) {
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    if (dc.xrow[2 * a] >= 0) {
                        h_a[dc.xslot(a)] = hx[a];
                        q_a[dc.xslot(a)] = sx[a];
                    }
            }
        }
        if (dc.jb[0] >= 0 && !bcand) ++n_st;
#pragma unroll
        for (int t = 0; t < kRB; ++t)
#pragma unroll
            for (int q = 0; q < PER; ++q) V::axpy(bcand ? 0.f : hv[t], cur.dn[t][q], acc[q]);  // (no down row: dummy)
        if (xkind == 2) {
#pragma unroll
            for (int a = 0; a < kXL; ++a) {
                // an empty slot read the dummy vector: its weight is zero
                const float hd = dc.xrow[a] >= 0 ? h_a[dc.xslot(a)] : 0.f;
#pragma unroll
                for (int q = 0; q < PER; ++q) V::axpy(hd, cur.xl[a][q], acc_sel[q]);
            }
        }
        if (dc.last_a()) {
            // Publish this workgroup's candidate results: one tagged word each, written through, so the hand-over
            // needs no cache write-back, no acknowledgement and no counter.  h_a was written by thread 0 of this
            // same wave, and a wave's LDS operations execute in order.
            if (wave == 0 && lane < n_aslots) {
                const float hvv = h_a[lane];
                // (what the selector ranks: h, from which it forms n_j |h_j|, or the input-side score itself)
                coherent_store(&p.hc[lane * n_wg + b], tagged(__float_as_uint(input_side ? q_a[lane] : hvv), epoch));
                p.h[j_a[lane]] = hvv;
            }
            POP_STAMP(1);
        }
        if (n_st == kKeep) flush_hidden();
    };

    RoundBuf<V, PER> buf_a, buf_b;  // ping-pong: one is reduced while the other's loads are in flight
#pragma unroll
    for (int a = 0; a < kXL; ++a)
#pragma unroll
        for (int q = 0; q < PER; ++q) buf_a.xl[a][q] = buf_b.xl[a][q] = V::zero();  // read before the first extra rows
    RoundDesc d0, d1, d2;           // descriptors of the round being reduced, the one in flight, the one after
    make_desc(d0);
    load_round<V, PER>(buf_a, d0, w, nvec, col, ok);
    make_desc(d1);
    int i = 0;
    // a round without work can still be followed by one with work (selected rows, once the selection is known)
    while (d0.work || d1.work) {
        step(buf_a, d0, buf_b, d1, d2, i, std::integral_constant<int, 0>{});
        ++i;
        d0 = d1;
        d1 = d2;
        if (!(d0.work || d1.work)) break;
        step(buf_b, d0, buf_a, d1, d2, i, std::integral_constant<int, 1>{});
        ++i;
        d0 = d1;
        d1 = d2;
    }
    POP_STAMP(2);

    // Adds the down rows of the selected slots in rem_d (this workgroup's own candidates; h still in LDS).
    auto drain_selected = [&]() {
        while (rem_d) {
            // eight rows per trip to memory (both round buffers are free by now)
            int sl[2 * kXL];
            uint32_t off[2 * kXL];
#pragma unroll
            for (int a = 0; a < 2 * kXL; ++a) {
                sl[a] = -1;
                off[a] = 0;
                if (rem_d) {
                    sl[a] = __builtin_ctz(rem_d);
                    rem_d &= rem_d - 1;
                    off[a] = ((uint32_t)uniform(j_a[sl[a]]) * 3u + 2u) * (uint32_t)nvec;
                }
            }
#pragma unroll
            for (int a = 0; a < 2 * kXL; ++a)
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const vec_t v = w[(ok[q] && sl[a] >= 0) ? off[a] + (uint32_t)col[q] : 0u];
                    if (a < kXL)
                        buf_a.xl[a][q] = v;
                    else
                        buf_b.xl[a - kXL][q] = v;
                }
#pragma unroll
            for (int a = 0; a < 2 * kXL; ++a) {
                const float hd = sl[a] >= 0 ? h_a[sl[a]] : 0.f;  // an empty slot read a dummy vector: weight zero
#pragma unroll
                for (int q = 0; q < PER; ++q) V::axpy(hd, a < kXL ? buf_a.xl[a][q] : buf_b.xl[a - kXL][q], acc_sel[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < PER; ++q)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[q][e] += acc_sel[q][e];
    };

    // This workgroup's partial y: one row of float32, summed with the others' by decode_tail_kernel.  (Summing the
    // rows inside this launch was built twice - behind an arrival counter, and with every element a tagged word that
    // the readers wait for - and measured no faster than the second launch: after the slowest workgroup's last store
    // either form needs the store to become visible, a look that finds it and a trip for the rows, while the launch
    // boundary is one kernel start plus one trip.)  The last workgroup to get here starts the next epoch: everybody
    // has stopped looking at this one's words.
    auto store_partial = [&]() __attribute__((always_inline)) {
        float *dst = p.partial + (size_t)b * p.d;
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (ok[q]) {
#pragma unroll
                for (int e = 0; e < E; e += 4)
                    *reinterpret_cast<float4 *>(dst + (size_t)col[q] * E + e) =
                        make_float4(acc[q][e], acc[q][e + 1], acc[q][e + 2], acc[q][e + 3]);
            }
        if (tid == 0 && atomicAdd(&p.ctr[1], 1) == n_wg - 1) {
            coherent_store(&p.ctr[1], 0);
            coherent_store(&p.ctr[0], epoch + 1);
        }
    };

    if (b == 0) {
        // ---- select (workgroup 0 only): collect every candidate's h (tagged words; bounded wait), form the step
        // scores I_j(t) = n_j |h_j| (Eq. 3 with one token), then top-k
        for (int q = tid; q < n_wg; q += blockDim.x) wg_bits[q] = 0;
        const int n_cand = p.n_cand;
        const bool in_lds = n_cand <= kSelLdsKeys;
        bool got_all = true;
        for (int base = 0; base < n_cand; base += 4 * blockDim.x) {
            unsigned long long v[4];
            int c[4], j[4];
            float nr[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                c[u] = base + u * blockDim.x + tid;
                j[u] = c[u] < n_cand ? p.cand_idx[c[u]] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) nr[u] = p.nrm[j[u]];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = c[u] < n_cand ? coherent_load(&p.hc[c[u]]) : tagged(0, epoch);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                for (int it = 0; (int)(v[u] >> 32) != epoch && it < limit; ++it) {
                    __builtin_amdgcn_s_sleep(2);
                    v[u] = coherent_load(&p.hc[c[u]]);
                }
                if ((int)(v[u] >> 32) != epoch) got_all = false;
                if (c[u] < n_cand) {
                    const float hq = __uint_as_float((uint32_t)v[u]);
                    const float sc = input_side ? hq : nr[u] * fabsf(hq);
                    if (in_lds) {
                        sh.keys[c[u]] = score_key(sc);
                        p.cscore[c[u]] = sc;
                    } else {
                        coherent_store(&p.cscore[c[u]], sc);  // read back below by other threads of this workgroup
                    }
                }
            }
        }
        if (!got_all) p.ctr[2] = 1;
        if (!in_lds) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        POP_STAMP(3);
        block_select_candidates<true>(
            p.cscore, p.cand_idx, p.n_cand, p.k, p.mask, p.active_idx + p.n_ret, sh,
            [&](int c) { atomicOr(&wg_bits[c % n_wg], 1 << (c / n_wg)); },  // candidate c is slot c / n_wg of workgroup c % n_wg
            [&]() {  // publish the per-workgroup slot masks first: they are all the other workgroups wait for
                __syncthreads();
                for (int q = 1 + tid; q < n_wg && q < p.n_cand; q += blockDim.x)
                    coherent_store(&p.selw[(size_t)q * kSelStride], tagged((uint32_t)wg_bits[q], epoch));
            },
#ifdef POP_TRACE
            p.trace ? p.trace + 1023 * 8 : nullptr,
#else
            nullptr,
#endif
            nullptr, 1, in_lds);
        if (tid == 0 && p.n_active) *p.n_active = p.n_ret + p.k;
        POP_STAMP(4);
        bits_known = true;
        rem_d = wg_bits[0];
        drain_selected();
        store_partial();
        POP_STAMP(6);
        return;
    }

    // ---- selected candidates of this worker that did not ride along with the retained rounds
    if (n_aslots > 0) {
        if (!bits_known) {
            // normally the word arrived during the retained rounds; else wait (bounded)
            if (tid == 0) {
                unsigned long long v = coherent_load(my_word);
                for (int it = 0; (int)(v >> 32) != epoch && it < limit; ++it) {
                    __builtin_amdgcn_s_sleep(2);
                    v = coherent_load(my_word);
                }
                const bool here = (int)(v >> 32) == epoch;
                if (!here) p.ctr[2] = 1;  // the step is flagged invalid; it goes on without this workgroup's selection
                s_flag = here ? (int)(uint32_t)v : 0;
            }
            __syncthreads();
            bits_known = true;
            rem_d = s_flag;
        }
        POP_STAMP(3);
    }
    drain_selected();
    POP_STAMP(4);
    __syncthreads();
    for (int e = tid; e < n_st * kRB; e += blockDim.x)
        if (j_st[e] >= 0) p.h[j_st[e]] = h_st[e];
    store_partial();
    POP_STAMP(6);
}

// y[o] = sum over workgroups (in order) of partial[b][o].  A workgroup owns 64 outputs; its 16 waves each sum a
// contiguous sixteenth of the partial rows (independent loads, fixed order) and wave 0 combines them in wave order,
// so y does not depend on scheduling.
constexpr int kTailWaves = 16;
__global__ __launch_bounds__(1024) void decode_tail_kernel(const float *__restrict__ partial, int n_wg, int d,
                                                           void *__restrict__ y, int y_bf16)
{
    __shared__ float part[kTailWaves][kWave];
    const int lane = threadIdx.x % kWave, q = threadIdx.x / kWave;
    const int o = blockIdx.x * kWave + lane;
    const int per = (n_wg + kTailWaves - 1) / kTailWaves;
    const int s0 = min(n_wg, q * per), s1 = min(n_wg, q * per + per);
    float acc = 0.f;
    if (o < d) {
        int s = s0;
        for (; s + 16 <= s1; s += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = partial[(size_t)(s + u) * d + o];
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += v[u];
        }
        for (; s < s1; ++s) acc += partial[(size_t)s * d + o];
    }
    part[q][lane] = acc;
    __syncthreads();
    if (q == 0 && o < d) {
        float v = 0.f;
#pragma unroll
        for (int u = 0; u < kTailWaves; ++u) v += part[u][lane];
        if (y_bf16)
            ((uint16_t *)y)[o] = f32_to_bf16(v);
        else
            ((float *)y)[o] = v;
    }
}

// ---------------------------------------------------------------- host side
// The kernel is built for two workgroup size limits: up to 512 threads (twice the registers per thread, enough for
// two vector columns per thread without spilling) and up to 1024.
template <class V, int PER, int MAXB>
static hipError_t fused_launch(const FusedPlan &pl, FusedParams &p, hipStream_t s)
{
    hipLaunchKernelGGL((decode_fused_kernel<V, PER, MAXB>), dim3(pl.n_wg), dim3(pl.block), 0, s, p);
    return hipGetLastError();
}

template <class V, int PER, int MAXB>
static hipError_t fused_occupancy(int block, int *blocks_per_cu)
{
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_fused_kernel<V, PER, MAXB>, block, 0);
}

// Calls fn.template operator()<V, PER, MAXB>() for the plan's variant.
template <class Fn>
static hipError_t fused_dispatch(int is_bf16, int per, int block, Fn fn)
{
    const bool small = block <= 512;
    if (is_bf16) {
        if (per == 1) return small ? fn.template operator()<VecBF16, 1, 512>() : fn.template operator()<VecBF16, 1, 1024>();
        return small ? fn.template operator()<VecBF16, 2, 512>() : fn.template operator()<VecBF16, 2, 1024>();
    }
    if (per == 1) return small ? fn.template operator()<VecF32, 1, 512>() : fn.template operator()<VecF32, 1, 1024>();
    return small ? fn.template operator()<VecF32, 2, 512>() : fn.template operator()<VecF32, 2, 1024>();
}

struct FusedOccupancyFn {
    int block;
    int *blocks_per_cu;
    template <class V, int PER, int MAXB>
    hipError_t operator()() const
    {
        return fused_occupancy<V, PER, MAXB>(block, blocks_per_cu);
    }
};
struct FusedLaunchFn {
    const FusedPlan &pl;
    FusedParams &p;
    hipStream_t s;
    template <class V, int PER, int MAXB>
    hipError_t operator()() const
    {
        return fused_launch<V, PER, MAXB>(pl, p, s);
    }
};

int fused_max_workgroups() { return 1024; }
size_t fused_selw_words() { return (size_t)1024 * kSelStride; }

// Chooses the launch shape; false when the fused kernel does not support this shape.
bool fused_plan(int d, int is_bf16, int n_ret, int n_cand, int wg_target, FusedPlan *pl)
{
    const int E = is_bf16 ? 8 : 4, nvec = d / E;
    // one vector column per thread up to 512 threads, then two (a workgroup of up to 512 threads has twice the
    // registers per thread); POP_FUSED_PER=1 / 2 overrides for 128 <= d/E <= 1024 (tuning)
    int per = nvec > 512 ? 2 : 1;
    if (nvec <= 1024 && nvec >= 128)
        if (const char *e = getenv("POP_FUSED_PER")) per = atoi(e) == 1 ? 1 : 2;
    if (nvec > 2048) return false;
    pl->per = per;
    pl->block = ((nvec + per * kWave - 1) / (per * kWave)) * kWave;
    const int rounds_total = (n_ret + kRB - 1) / kRB;
    int workers = rounds_total;
    if ((n_cand + 1) / 2 > workers) workers = (n_cand + 1) / 2;
    if (workers < 1) workers = 1;
    if (workers > wg_target - 1) workers = wg_target - 1;
    pl->n_wg = workers + 1;
    // a workgroup's candidate slots must fit its selection word, its retained rounds the staged list
    if ((n_cand + pl->n_wg - 1) / pl->n_wg > kMaxASlots) return false;
    pl->n_static = (rounds_total + workers - 1) / workers;
    return pl->n_static <= kMaxStatic;
}

hipError_t fused_resident_limit(int is_bf16, const FusedPlan &pl, int n_cu, int *max_wg)
{
    int per_cu = 0;
    hipError_t e = fused_dispatch(is_bf16, pl.per, pl.block, FusedOccupancyFn{pl.block, &per_cu});
    if (e != hipSuccess) return e;
    *max_wg = per_cu * n_cu;
    return hipSuccess;
}

hipError_t launch_decode_fused(const FusedPlan &pl, int is_bf16, FusedParams &p, hipStream_t s)
{
    p.n_static = pl.n_static;
    return fused_dispatch(is_bf16, pl.per, pl.block, FusedLaunchFn{pl, p, s});
}

hipError_t launch_decode_tail(const float *partial, int n_wg, int d, void *y, int y_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(decode_tail_kernel, dim3((d + kWave - 1) / kWave), dim3(kTailWaves * kWave), 0, s, partial, n_wg, d,
                       y, y_bf16);
    return hipGetLastError();
}

}  // namespace pop
