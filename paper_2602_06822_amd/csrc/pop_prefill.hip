// Prefill: gate/up contraction over all m channels and all T prompt tokens, fused with the column-wise
// importance reduction  s2[j] = sum_t H[t][j]^2  (Sec. 3.3 "Prefilling Stage"; Eq. 3: activation norm over
// tokens and samples).  In its plain form H is never written to memory.
//
// bf16: MFMA 32x32x16 tiles.  A workgroup owns BM tokens (256 with 8 waves, 4 along the tokens x 2 along the B rows;
// 128 with 4 waves for short prompts) and a chunk of up to 96 channels, i.e. up to 192 rows of the B operand (gate
// and up rows of the channel-major blocks w[j] = [gate row | up row | down column]); a wave owns 64 tokens x 48
// channels = 96 B rows.  The 96 B rows of a wave are three fragments: gate of its channels 0..31, up of the same
// channels (same lane and register slot in the two accumulators, so silu(g)*u needs no exchange), and a mixed
// fragment [gate 32..47 | up 32..47] whose halves meet through one cross-lane move in the epilogue.  A second
// tile form drops the mixed fragment (64 channels per chunk, 64 B rows per wave).  The chunk size is chosen so
// that the tiles divide evenly over the compute units (one or a whole number of tiles each).  Each accumulator
// lane holds 16 token rows of one channel column, so the token reduction is in-register adds, one cross-half
// shuffle and an LDS combine of the token waves.  Token tiles write separate partial rows that are summed in
// tile order.  Operand rows that are whole k-steps long (d a multiple of 64) go from global memory straight into LDS
// (global_load_lds, 1 KB = 8 unpadded rows per wave instruction, 16-byte units XOR-swizzled by row pair so that the
// fragment reads stay conflict-free); fetching them through registers costs a quarter more time even when every load
// hits the cache, and remains the path for other row lengths.  On the direct path every wave issues the same loads
// in every k-step (rows that do not exist are pointed at one that does and left out by the epilogue), so a step waits
// with an exact count for its own rows only, and the 128-token tile runs a ring of three LDS buffers: short prompts
// are bound by the weight stream from memory, where two k-steps in flight carry twice the bytes of one.
// Two more forms of the same kernel serve the forward pass of a whole prompt under the pruning structure
// (Sec. 3.4): one also writes H (rounded to bf16) as [T][m]; one runs its chunks over a device-resident list of
// active channels instead of all m and writes H (optionally times a per-token mask) in compact form
// [T][list position] for the down projection instead of reducing its squares.
// float32: plain FMA tiles with the same structure (64 tokens x 32 channels per workgroup).
#include <stdlib.h>

#include "pop_internal.h"

namespace pop {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kPfBMmin = 128;     // smallest token tile (sizes the partial-row buffer)
constexpr int kPfChunk = 96;      // channels per workgroup tile at most
constexpr int kPfBK = 64;         // k elements per stage
constexpr int kPfLd = kPfBK + 8;  // padded LDS row stride in elements (144 B): conflict-free 16-byte reads

constexpr int kPf32BM = 64;
constexpr int kPf32BC = 32;
constexpr int kPf32BK = 16;

int prefill_num_tiles(int T, int is_bf16)
{
    return is_bf16 ? (T + kPfBMmin - 1) / kPfBMmin : (T + kPf32BM - 1) / kPf32BM;
}

// Workgroups are dealt round-robin to the 8 XCDs; renumber so that consecutive logical tiles (the token tiles
// of one channel chunk, which share the weight rows) land on the same XCD and meet in its L2.
__device__ __forceinline__ int xcd_logical_block(int bid, int per_xcd) { return (bid % 8) * per_xcd + bid / 8; }

// Channel (relative to the chunk) and matrix (0 gate, 1 up) of B row r of the workgroup tile.  A wave owns NF
// fragments of 32 rows: gate and up of its channels 0..31 and, with NF = 3, the mixed fragment of channels 32..47.
template <int NF>
__device__ __forceinline__ void pf_row_channel(int r, int &ch, int &which)
{
    const int half = r / (NF * 32), rr = r % (NF * 32);
    if (rr < 64) {
        ch = half * (NF * 16) + rr % 32;
        which = rr / 32;
    } else {
        ch = half * 48 + 32 + rr % 16;
        which = (rr - 64) / 16;
    }
}

// Tile geometry: channel chunks of at most 96 channels (three fragments per wave) or at most 64 (two fragments), as
// many as make the tiles a whole number per compute unit; of the two forms the one that is cheaper on the busiest
// compute unit.  The kernel is bound by its LDS fragment reads, so a tile's cost is taken as the reads per k-slice
// of a wave: 2 token fragments + the B fragments (measured: a two-fragment tile takes 0.8 of a three-fragment one).
// Host and device share this because the list form learns its channel count on the device.
struct PfGeom {
    int chunk, n_ct, total, per_xcd, nf;
};
__host__ __device__ inline PfGeom prefill_geometry_nf(int n_ch, int n_tt, int n_cu, int nf)
{
    PfGeom g;
    g.nf = nf;
    const int cap = nf * 32;
    const int min_ct = (n_ch + cap - 1) / cap;
    const int per_cu = (min_ct * n_tt + n_cu - 1) / n_cu;
    int n_ct = per_cu * n_cu / n_tt;
    if (n_ct < min_ct) n_ct = min_ct;
    if (n_ct > n_ch) n_ct = n_ch;
    g.chunk = (n_ch + n_ct - 1) / n_ct;
    g.n_ct = (n_ch + g.chunk - 1) / g.chunk;
    g.total = n_tt * g.n_ct;
    g.per_xcd = (g.total + 7) / 8;
    return g;
}
__host__ __device__ inline PfGeom prefill_geometry(int n_ch, int n_tt, int n_cu)
{
    if (n_ch <= 0) return PfGeom{1, 0, 0, 0, 3};
    const PfGeom g3 = prefill_geometry_nf(n_ch, n_tt, n_cu, 3), g2 = prefill_geometry_nf(n_ch, n_tt, n_cu, 2);
    const int cost3 = (g3.total + n_cu - 1) / n_cu * 5, cost2 = (g2.total + n_cu - 1) / n_cu * 4;
    return cost2 < cost3 ? g2 : g3;
}

// silu(g) * u for the tile epilogue (96 values per lane, with no other tile to hide behind): hardware exp2 and
// reciprocal, each good to one unit in the last place, instead of the library exponential and the exact quotient
// (a fifth of the instructions).  g -> -inf gives g * 0, g -> +inf gives g * 1.
__device__ __forceinline__ float silu_mul_tile(float g, float u)
{
    const float e = __builtin_amdgcn_exp2f(g * -1.44269504088896341f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// What the list form adds to the plain prefill arguments.
struct PfStore {
    const int *list;            // active channels, ascending
    const int *n_list;          // their number (device)
    uint16_t *hc;               // [T][ldh] bf16: H of list position c in column c
    int ldh;
    const unsigned char *tmask; // per-token masks [T][m], or null
    int n_cu;
    // scores formed in the same launch (modes 0 and 2; null = leave that to the caller): the token tile of a
    // channel chunk that finishes last sums the chunk's partial rows
    int *fin_ctr = nullptr;     // one arrival counter per channel chunk; zero between launches
    const float *nrm = nullptr; // [m]
    float *scores = nullptr;    // [m]
};

// kMode 0: scores only (s2_part).  1: channels from st.list, H stored compact (no s2_part).  2: all m channels,
// s2_part and H stored as [T][m padded].
template <int BM, int NW, int NF, int kMode, bool kDma = false, int NS = 2>
__global__ __launch_bounds__(NW * 64) void prefill_bf16_kernel(const uint16_t *__restrict__ w,
                                                           const uint16_t *__restrict__ x, int T, int d, int m,
                                                           int n_ttiles, int chunk, int n_items, int per_xcd,
                                                           float *__restrict__ s2_part, PfStore st)
{
    constexpr int TW = NW / 2;          // waves along the tokens (2 along the B rows)
    constexpr int MT = BM / (32 * TW);  // 32-token fragments per wave
    constexpr int RP = NW * 8;          // rows one staging pass of the workgroup covers
    constexpr int BR = NF * 64;         // B rows of the workgroup tile
    constexpr int WC = NF * 16;         // channels per wave
    // LDS rows: 64 elements padded to 72 (register staging), or exactly 64 with the 16-byte units of row r stored
    // at unit ^ ((r / 2) % 8) (direct global -> LDS loads, which fill 1 KB = 8 whole rows per wave instruction)
    constexpr int LD = kDma ? kPfBK : kPfLd;
    extern __shared__ __attribute__((aligned(16))) uint16_t pf_lds[];
    static_assert(kDma || NS == 2, "the register-staged path has two LDS buffers");
    uint16_t *As = pf_lds;                    // [NS][BM * LD]
    uint16_t *Bs = pf_lds + NS * BM * LD;     // [NS][BR * LD]
    __shared__ float colsum[TW][kPfChunk];

    constexpr bool kList = kMode == 1, kStore = kMode != 0;
    int n_ch = m;  // channels the chunks run over
    if (kList) {
        n_ch = *st.n_list;
        const PfGeom g = prefill_geometry(n_ch, n_ttiles, st.n_cu);
        if (g.nf != NF) return;  // the other instantiation runs this list length
        chunk = g.chunk, n_items = g.total, per_xcd = g.per_xcd;
        if ((int)blockIdx.x >= per_xcd * 8) return;  // the grid was sized for the longest list
    }
    const int logical = xcd_logical_block(blockIdx.x, per_xcd);
    if (logical >= n_items) return;
    const int ctile = logical / n_ttiles, ttile = logical % n_ttiles;
    const int t0 = ttile * BM, c0 = ctile * chunk;
    const int cn = min(chunk, n_ch - c0);  // channels in this chunk

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int wm = wave / 2, wn = wave % 2;  // wave tile: tokens wm*BM/TW.., B rows wn*NF*32..

    // global -> LDS staging: 8 vectors of 16 bytes per 64-element row; the workgroup covers RP rows per pass
    const int ld_row = tid / 8, ld_kv = tid % 8;
    constexpr int PA = BM / RP, PB = BR / RP;
    static_assert(BM % RP == 0 && BR % RP == 0, "whole staging passes");
    uint4 ra[PA], rb[PB];
    // Row starts.  Register-staged path: null for a row of zeros (tokens beyond T, channels beyond the chunk).  Direct
    // path: such rows are pointed at a row that exists instead, so that every wave issues the same number of loads per
    // k-step (its waits count them); what they produce is left out by the epilogue.
    const uint16_t *pa[PA], *pb[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int t = t0 + ld_row + p * RP;
        pa[p] = kDma ? x + (size_t)min(t, T - 1) * d : (t < T ? x + (size_t)t * d : nullptr);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int ch, which;
        pf_row_channel<NF>(ld_row + p * RP, ch, which);
        if (ch < cn || kDma) {
            const int cc = min(ch, cn - 1);
            const int j = kList ? st.list[c0 + cc] : c0 + cc;
            pb[p] = w + ((size_t)j * 3 + which) * d;
        } else {
            pb[p] = nullptr;
        }
    }
    auto load_global = [&](int k0) {
        const int k = k0 + ld_kv * 8;
        const bool k_ok = k < d;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            ra[p] = (k_ok && pa[p]) ? *reinterpret_cast<const uint4 *>(pa[p] + k) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int p = 0; p < PB; ++p)
            rb[p] = (k_ok && pb[p]) ? *reinterpret_cast<const uint4 *>(pb[p] + k) : make_uint4(0, 0, 0, 0);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PA; ++p)
            *reinterpret_cast<uint4 *>(&As[(buf * BM + ld_row + p * RP) * LD + ld_kv * 8]) = ra[p];
#pragma unroll
        for (int p = 0; p < PB; ++p)
            *reinterpret_cast<uint4 *>(&Bs[(buf * BR + ld_row + p * RP) * LD + ld_kv * 8]) = rb[p];
    };
    // direct loads: this lane's 16 bytes land at LDS unit ld_kv of row ld_row of the pass, so it fetches the k-vector
    // that belongs there under the swizzle
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int src_kv = (ld_kv ^ ((ld_row / 2) % 8)) * 8;  // (passes are RP rows apart, a multiple of 16: same swizzle term)
    auto dma_load = [&](int buf, int k0) {
        typedef __attribute__((address_space(3))) void lds_t;
        typedef __attribute__((address_space(1))) const void glb_t;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            __builtin_amdgcn_global_load_lds((glb_t *)(pa[p] + k0 + src_kv),
                                             (lds_t *)(As + (buf * BM + p * RP + wave_u * 8) * LD), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < PB; ++p)
            __builtin_amdgcn_global_load_lds((glb_t *)(pb[p] + k0 + src_kv),
                                             (lds_t *)(Bs + (buf * BR + p * RP + wave_u * 8) * LD), 16, 0, 0);
    };

    f32x16_t acc[MT][NF];  // [token fragment][0 = gate 0..31, 1 = up 0..31, 2 = gate 32..47 | up 32..47]
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][f][v] = 0.f;

    const int n_k = (d + kPfBK - 1) / kPfBK;
    const int arow = wm * (BM / TW) + (lane % 32), brow = wn * (NF * 32) + (lane % 32), koff = (lane / 32) * 8;
    const int a_sw = (arow / 2) % 8, b_sw = (brow / 2) % 8;  // (fragments are 32 rows apart: same swizzle term)
    auto multiply = [&](int buf) {
        const uint16_t *Ab = As + (buf * BM + arow) * LD + (kDma ? 0 : koff);
        const uint16_t *Bb = Bs + (buf * BR + brow) * LD + (kDma ? 0 : koff);
        // the fragments of k-slice q + 1 are requested before the products of slice q are issued (two register
        // sets), so that their LDS latency runs under the matrix pipe
        bf16x8_t bf[2][NF], af[2][MT];
        auto fetch = [&](int q, int set) {
            // element offset of this lane's 8 k-values within its row
            const int ka = kDma ? (((q * 2 + lane / 32) ^ a_sw) * 8) : q * 16;
            const int kb = kDma ? (((q * 2 + lane / 32) ^ b_sw) * 8) : q * 16;
#pragma unroll
            for (int f = 0; f < NF; ++f) bf[set][f] = *reinterpret_cast<const bf16x8_t *>(Bb + f * 32 * LD + kb);
#pragma unroll
            for (int a = 0; a < MT; ++a) af[set][a] = *reinterpret_cast<const bf16x8_t *>(Ab + a * 32 * LD + ka);
        };
        fetch(0, 0);
#pragma unroll
        for (int q = 0; q < kPfBK / 16; ++q) {
            if (q + 1 < kPfBK / 16) fetch(q + 1, (q + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < MT; ++a)
#pragma unroll
                for (int f = 0; f < NF; ++f)
                    acc[a][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[q & 1][a], bf[q & 1][f], acc[a][f], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (kDma) {
        // (needs d % 64 == 0.)  A ring of NS LDS buffers: step ks multiplies buffer ks % NS while the rows of steps
        // ks + 1 .. ks + NS - 1 are landing in or on their way to the others.  Per step: wait until this wave's loads
        // of step ks have landed (all but the (NS - 2) (PA + PB) younger ones), meet the other waves (now everybody's
        // have, and everybody is done reading the buffer of step ks - 1), request step ks + NS - 1 into that buffer,
        // multiply.  Steps beyond the last are requested again from the last step's columns, so the count holds.
        constexpr int kYounger = (NS - 2) * (PA + PB);
        static_assert(kYounger < 64, "vmcnt is a 6-bit counter");
        // s_waitcnt with only the vector-memory counter set: vmcnt[3:0] | expcnt 7 << 4 | lgkmcnt 15 << 8 | vmcnt[5:4] << 14
        constexpr int kWaitImm = (kYounger & 15) | (7 << 4) | (15 << 8) | ((kYounger >> 4) << 14);
#pragma unroll
        for (int q = 0; q < NS - 1; ++q) dma_load(q, min(q, n_k - 1) * kPfBK);
        for (int ks = 0; ks < n_k; ++ks) {
            __builtin_amdgcn_s_waitcnt(kWaitImm);
            asm volatile("s_barrier" ::: "memory");  // (no fence: a fence would wait for the younger loads too)
            dma_load((ks + NS - 1) % NS, min(ks + NS - 1, n_k - 1) * kPfBK);
            multiply(ks % NS);
        }
        __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8));  // the surplus requests, before LDS is reused
        __syncthreads();
    } else {
        // step ks multiplies LDS buffer ks % 2 while the rows of step ks + 1 are on their way through registers
        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int ks = 0; ks < n_k; ++ks) {
            const int buf = ks & 1;
            if (ks + 1 < n_k) load_global((ks + 1) * kPfBK);
            multiply(buf);
            if (ks + 1 < n_k) store_lds(buf ^ 1);
            __syncthreads();
        }
    }

    // epilogue: lane holds 16 * MT token rows of column (lane % 32) of each fragment.  Register-staged path: rows of
    // padded tokens and columns of padded channels are exactly 0.  Direct path: they hold products of the rows their
    // loads were pointed at; padded tokens are left out of the sums below, padded channels are never written.
    // H of the tile (modes 1 and 2), written after the partial sums have gone out: the tile's arrival is counted once
    // its partial row is acknowledged, and that wait should not take in the much larger H.
    auto store_h = [&]() {
        // register v of a fragment is token row (v / 4) * 8 + (lane / 32) * 4 + v % 4, column lane % 32
        const int col = lane % 32;
        const int c01 = wn * WC + col, c2 = wn * WC + 32 + col;
        const bool ok01 = c01 < cn, ok2 = NF == 3 && col < 16 && c2 < cn;
        const int j01 = (kList && st.tmask && ok01) ? st.list[c0 + c01] : 0;
        const int j2 = (kList && st.tmask && ok2) ? st.list[c0 + c2] : 0;
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + wm * (BM / TW) + a * 32 + (v / 4) * 8 + (lane / 32) * 4 + v % 4;
                float h01 = silu_mul_tile(acc[a][0][v], acc[a][1][v]);
                float h2 = 0.f;
                if (NF == 3) {
                    const float g2 = acc[a][NF - 1][v];
                    const float u2 = __shfl_xor(g2, 16, kWave);
                    h2 = silu_mul_tile(g2, u2);
                }
                if (t < T) {
                    uint16_t *row = st.hc + (size_t)t * st.ldh + c0;
                    if (ok01) {
                        if (kList && st.tmask && !st.tmask[(size_t)t * m + j01]) h01 = 0.f;
                        row[c01] = f32_to_bf16(h01);
                    }
                    if (ok2) {
                        if (kList && st.tmask && !st.tmask[(size_t)t * m + j2]) h2 = 0.f;
                        row[c2] = f32_to_bf16(h2);
                    }
                }
            }
    };
    if (kList) {
        store_h();
        return;
    }
    float ss01 = 0.f, ss2 = 0.f;
    const int t_left = T - (t0 + wm * (BM / TW) + (lane / 32) * 4);  // this lane's rows below t_left are tokens
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const bool live = !kDma || a * 32 + (v / 4) * 8 + v % 4 < t_left;
            const float hv = silu_mul_tile(acc[a][0][v], acc[a][1][v]);
            ss01 = fmaf(hv, live ? hv : 0.f, ss01);
            if (NF == 3) {
                // mixed fragment: the up value of column c < 16 sits in lane c + 16, same register
                const float g2 = acc[a][NF - 1][v];
                const float u2 = __shfl_xor(g2, 16, kWave);
                const float h2 = silu_mul_tile(g2, u2);
                ss2 = fmaf(h2, live ? h2 : 0.f, ss2);
            }
        }
    ss01 += __shfl_xor(ss01, 32, kWave);
    ss2 += __shfl_xor(ss2, 32, kWave);
    if (lane < 32) colsum[wm][wn * WC + lane] = ss01;
    if (NF == 3 && lane < 16) colsum[wm][wn * WC + 32 + lane] = ss2;
    __syncthreads();
    if (tid < cn) {
        float tot = 0.f;
#pragma unroll
        for (int q = 0; q < TW; ++q) tot += colsum[q][tid];
        if (st.fin_ctr)
            coherent_store(&s2_part[(size_t)ttile * m + c0 + tid], tot);
        else
            s2_part[(size_t)ttile * m + c0 + tid] = tot;
    }
    if (st.fin_ctr) {
        // Scores of this chunk's channels (Eq. 3): I_j = n_j * sqrt(sum over the token tiles, in tile order and in
        // double, of the partial sums).  The partial rows are written through and read with device-coherent loads;
        // a tile counts itself in once its own row has been acknowledged, and the tile that completes the count does
        // the sum and puts the counter back to zero for the next launch.  Nobody waits for anybody.
        __shared__ int fin_last;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const bool last = atomicAdd(&st.fin_ctr[ctile], 1) == n_ttiles - 1;
            if (last) coherent_store(&st.fin_ctr[ctile], 0);
            fin_last = last;
        }
        __syncthreads();
        if (fin_last && tid < cn) {
            double acc = 0.0;
            for (int t = 0; t < n_ttiles; ++t) acc += (double)coherent_load(&s2_part[(size_t)t * m + c0 + tid]);
            st.scores[c0 + tid] = (float)((double)st.nrm[c0 + tid] * sqrt(acc));
        }
    }
    if (kStore) store_h();
}

// float32: 64 tokens x 32 channels per workgroup; thread (tx = channel, ty = group of 8 tokens).
__global__ __launch_bounds__(256) void prefill_f32_kernel(const float *__restrict__ w, const float *__restrict__ x,
                                                          int T, int d, int m, float *__restrict__ s2_part)
{
    __shared__ float As[kPf32BM][kPf32BK + 1];
    __shared__ float Bg[kPf32BC][kPf32BK + 1];
    __shared__ float Bu[kPf32BC][kPf32BK + 1];
    __shared__ float colsum[8][kPf32BC];
    const int c0 = blockIdx.x * kPf32BC, ttile = blockIdx.y, t0 = ttile * kPf32BM;
    const int tid = threadIdx.x, tx = tid % 32, ty = tid / 32;
    float g[8], u[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) g[i] = u[i] = 0.f;
    for (int k0 = 0; k0 < d; k0 += kPf32BK) {
        for (int i = tid; i < kPf32BM * kPf32BK; i += 256) {
            int r = i / kPf32BK, k = i % kPf32BK;
            As[r][k] = (t0 + r < T && k0 + k < d) ? x[(size_t)(t0 + r) * d + k0 + k] : 0.f;
        }
        for (int i = tid; i < kPf32BC * kPf32BK; i += 256) {
            int r = i / kPf32BK, k = i % kPf32BK;
            bool ok = c0 + r < m && k0 + k < d;
            Bg[r][k] = ok ? w[((size_t)(c0 + r) * 3) * d + k0 + k] : 0.f;
            Bu[r][k] = ok ? w[((size_t)(c0 + r) * 3 + 1) * d + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kPf32BK; ++k) {
            float wg = Bg[tx][k], wu = Bu[tx][k];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float a = As[ty * 8 + i][k];
                g[i] = fmaf(a, wg, g[i]);
                u[i] = fmaf(a, wu, u[i]);
            }
        }
        __syncthreads();
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float hv = silu_mul(g[i], u[i]);
        ss = fmaf(hv, hv, ss);
    }
    colsum[ty][tx] = ss;
    __syncthreads();
    if (tid < kPf32BC && c0 + tid < m) {
        float tot = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) tot += colsum[q][tid];
        s2_part[(size_t)ttile * m + c0 + tid] = tot;
    }
}

// Token tile: 256 or 128 tokens, whichever gives the cheaper schedule: tiles per compute unit on the busiest one
// (after the chunks are evened out) times a tile's measured relative cost - 1 for 256 tokens x three fragments, 0.8
// with two fragments, and 0.6 of either for the 128-token form (half the products, a ring of three LDS buffers).
// At config 2 this picks 128 up to 256 tokens and 256 from there on.  POP_PF_BM=128 / 256 overrides (tuning).
static int prefill_token_tile(int T, int n_ch, int n_cu)
{
    static const int forced = getenv("POP_PF_BM") ? atoi(getenv("POP_PF_BM")) : 0;
    if (forced == 128 || forced == 256) return forced;
    int best_bm = 256;
    long best = -1;
    for (int bm = 256; bm >= 128; bm -= 128) {
        const PfGeom g = prefill_geometry(n_ch, (T + bm - 1) / bm, n_cu);
        const long waves = (g.total + n_cu - 1) / n_cu;
        const long cost = waves * (g.nf == 3 ? 5 : 4) * (bm == 256 ? 5 : 3);
        if (best < 0 || cost < best) best = cost, best_bm = bm;
    }
    return best_bm;
}

int prefill_rows_used(int T, int is_bf16, int m, int n_cu)
{
    if (!is_bf16) return (T + kPf32BM - 1) / kPf32BM;
    const int bm = prefill_token_tile(T, m, n_cu);
    return (T + bm - 1) / bm;
}

template <int BM, int NW, int NF, int kMode>
static hipError_t launch_pf_bf16(int blocks, hipStream_t s, const void *w, const void *x, int T, int d, int m, int n_tt,
                                 const PfGeom &g, float *s2_part, const PfStore &st)
{
    // rows that are whole k-steps long go from global memory straight into LDS (POP_PF_DMA=0 keeps them on the
    // register-staged path, for comparison).  The 128-token tile is small enough for a ring of three LDS buffers:
    // short prompts are bound by the weight stream from memory, and two k-steps in flight per compute unit carry
    // twice the bytes of one.
    static const int use_dma = getenv("POP_PF_DMA") ? atoi(getenv("POP_PF_DMA")) : 1;
    if (use_dma && d % kPfBK == 0) {
        constexpr int NS = BM <= 128 ? 3 : 2;
        const size_t lds_d = (size_t)NS * (BM + NF * 64) * kPfBK * sizeof(uint16_t);
        hipError_t e =
            hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_bf16_kernel<BM, NW, NF, kMode, true, NS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_d);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((prefill_bf16_kernel<BM, NW, NF, kMode, true, NS>), dim3(blocks), dim3(NW * 64), lds_d, s,
                           (const uint16_t *)w, (const uint16_t *)x, T, d, m, n_tt, g.chunk, g.total, g.per_xcd, s2_part,
                           st);
        return hipGetLastError();
    }
    const size_t lds = (size_t)2 * (BM + NF * 64) * kPfLd * sizeof(uint16_t);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_bf16_kernel<BM, NW, NF, kMode>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((prefill_bf16_kernel<BM, NW, NF, kMode>), dim3(blocks), dim3(NW * 64), lds, s,
                       (const uint16_t *)w, (const uint16_t *)x, T, d, m, n_tt, g.chunk, g.total, g.per_xcd, s2_part, st);
    return hipGetLastError();
}

// Whether the contraction's launch forms the scores itself: when every compute unit runs one tile at most.  The tile
// that completes a chunk learns so through a write-through store, its acknowledgement and a counted arrival, a few
// microseconds that nothing hides at the end of a launch with one tile per compute unit anyway, but that would stand
// between the tiles a compute unit runs back to back on a long prompt (measured: +14 us at 2048 tokens).
static bool prefill_scores_in_launch(int is_bf16, int T, int m, int n_cu)
{
    if (!is_bf16 || T < 1) return false;
    const int bm = prefill_token_tile(T, m, n_cu);
    return prefill_geometry(m, (T + bm - 1) / bm, n_cu).total <= n_cu;
}

template <int kMode>
static hipError_t launch_pf_bf16_all(const void *w, int d, int m, const void *x, int T, float *s2_part, int n_cu,
                                     PfStore st, hipStream_t s)
{
    const int bm = prefill_token_tile(T, m, n_cu);
    const int n_tt = (T + bm - 1) / bm;
    const PfGeom g = prefill_geometry(m, n_tt, n_cu);
    const int blocks = g.per_xcd * 8;
    if (!prefill_scores_in_launch(1, T, m, n_cu)) st.fin_ctr = nullptr;
    // 256-token tiles run with 8 waves (two per SIMD: one wave's waits for staging loads, LDS writes and the
    // k-step barrier are covered by the other's products), 128-token tiles with 4
    if (bm == 256 && g.nf == 3) return launch_pf_bf16<256, 8, 3, kMode>(blocks, s, w, x, T, d, m, n_tt, g, s2_part, st);
    if (bm == 256) return launch_pf_bf16<256, 8, 2, kMode>(blocks, s, w, x, T, d, m, n_tt, g, s2_part, st);
    if (g.nf == 3) return launch_pf_bf16<128, 4, 3, kMode>(blocks, s, w, x, T, d, m, n_tt, g, s2_part, st);
    return launch_pf_bf16<128, 4, 2, kMode>(blocks, s, w, x, T, d, m, n_tt, g, s2_part, st);
}

// bf16 only: the prefill contraction that also keeps H, h_all[t][j] = bf16(H[t][j]) with row stride ldh.
hipError_t launch_prefill_gateup_keep_bf16(const void *w, int d, int m, const void *x, int T, float *s2_part,
                                           uint16_t *h_all, int ldh, int n_cu, hipStream_t s, const PrefillScores *fin)
{
    PfStore st{nullptr, nullptr, h_all, ldh, nullptr, n_cu};
    if (fin) st.fin_ctr = fin->chunk_ctr, st.nrm = fin->nrm, st.scores = fin->scores;
    return launch_pf_bf16_all<2>(w, d, m, x, T, s2_part, n_cu, st, s);
}

bool prefill_forms_scores(int is_bf16, int T, int m, int n_cu) { return prefill_scores_in_launch(is_bf16, T, m, n_cu); }

hipError_t launch_prefill_gateup(const void *w, int is_bf16, int d, int m, const void *x, int T, float *s2_part,
                                 int n_cu, hipStream_t s, const PrefillScores *fin)
{
    if (is_bf16) {
        PfStore st{};
        if (fin) st.fin_ctr = fin->chunk_ctr, st.nrm = fin->nrm, st.scores = fin->scores;
        return launch_pf_bf16_all<0>(w, d, m, x, T, s2_part, n_cu, st, s);
    }
    dim3 grid((m + kPf32BC - 1) / kPf32BC, (T + kPf32BM - 1) / kPf32BM);
    hipLaunchKernelGGL(prefill_f32_kernel, grid, dim3(256), 0, s, (const float *)w, (const float *)x, T, d, m, s2_part);
    return hipGetLastError();
}

// bf16 only.  Gate/up over the channels of a device-resident list; hc[t][c] = bf16(H[t][list[c]]) (times
// tmask[t][list[c]] if tmask is given).  The list's length is known on the device only: both tile forms are
// launched, each sized for the longest possible list (m channels), and the one the length does not call for exits
// at once.
hipError_t launch_gateup_list_bf16(const void *w, int d, int m, const void *x, int T, const int *list, const int *n_list,
                                   const unsigned char *tmask, uint16_t *hc, int ldh, int n_cu, hipStream_t s)
{
    const int bm = prefill_token_tile(T, m, n_cu);  // (the list's length is not known here: priced as all m channels)
    const int n_tt = (T + bm - 1) / bm;
    PfStore st{list, n_list, hc, ldh, tmask, n_cu};
    PfGeom g{};
    hipError_t e = hipSuccess;
    for (int nf = 3; nf >= 2 && e == hipSuccess; --nf) {
        // an upper bound of the tile count over all list lengths <= m (the count before chunks are evened out)
        const int min_ct = (m + nf * 32 - 1) / (nf * 32);
        const int per_cu = (min_ct * n_tt + n_cu - 1) / n_cu;
        int n_ct = per_cu * n_cu / n_tt;
        if (n_ct < min_ct) n_ct = min_ct;
        const int blocks = (n_tt * n_ct + 7) / 8 * 8;
        if (bm == 256 && nf == 3) e = launch_pf_bf16<256, 8, 3, 1>(blocks, s, w, x, T, d, m, n_tt, g, nullptr, st);
        else if (bm == 256) e = launch_pf_bf16<256, 8, 2, 1>(blocks, s, w, x, T, d, m, n_tt, g, nullptr, st);
        else if (nf == 3) e = launch_pf_bf16<128, 4, 3, 1>(blocks, s, w, x, T, d, m, n_tt, g, nullptr, st);
        else e = launch_pf_bf16<128, 4, 2, 1>(blocks, s, w, x, T, d, m, n_tt, g, nullptr, st);
    }
    return e;
}

// scores[j] = nrm[j] * sqrt(sum over token tiles, in tile order, of s2_part[tile][j])   (Eq. 3)
__global__ __launch_bounds__(256) void scores_from_partials_kernel(const float *__restrict__ s2_part, int n_tiles, int m,
                                                                   const float *__restrict__ nrm,
                                                                   float *__restrict__ scores)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    double acc = 0.0;
    for (int t = 0; t < n_tiles; ++t) acc += (double)s2_part[(size_t)t * m + j];
    scores[j] = (float)((double)nrm[j] * sqrt(acc));
}

hipError_t launch_scores_from_partials(const float *s2_part, int n_tiles, int m, const float *nrm, float *scores,
                                       hipStream_t s)
{
    hipLaunchKernelGGL(scores_from_partials_kernel, dim3((m + 255) / 256), dim3(256), 0, s, s2_part, n_tiles, m, nrm,
                       scores);
    return hipGetLastError();
}

}  // namespace pop
