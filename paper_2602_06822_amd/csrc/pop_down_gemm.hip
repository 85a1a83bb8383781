// Down projection of a whole prompt under the pruning structure (Sec. 3.4: the forward pass over the active channels):
//     Y[t][n] = sum over list positions c < a of  Hc[t][c] * W_down[n][list[c]],
// a K-gathered bf16 MFMA GEMM: the contraction runs over the a active channels, whose down columns are the rows
// w[list[c]][2][:] of the channel-major weights, contiguous along n.
//
// The matrix cores want both operands with the contraction index fastest inside a lane (8 consecutive k per lane for
// the 32x32x16 tile).  Hc is stored that way; the weight rows are not (n is contiguous, k jumps from row to row).
// They are staged into LDS as they come, [k][n], and fetched with the transposing LDS read of this chip: a block of
// 16 lanes points at a 4 (k) x 16 (n) patch, lane i at the 4 values of row i / 4 starting at column 4 (i % 4), and
// receives it transposed, lane j the 4 k-values of column j.  Two such reads make the 8 values of one B fragment.
//
// Workgroup: 256 tokens x 128 columns, 8 waves (4 along the tokens x 2 along n), wave tile 64 x 64 = 2 x 2 MFMA
// tiles, k-steps of 64 channels.  Short prompts do not give enough tiles to fill the chip, so the contraction is
// split into n_split ranges whose float32 partial results are summed, in split order, by a second kernel
// (deterministic).  Two kernels share this tile:
//  * down_gemm_dma_kernel (d a multiple of 128): both operands go from global memory straight into a ring of three
//    unpadded, swizzled LDS buffers, with one exact wait per k-step (described at the kernel);
//  * down_gemm_bf16_kernel (any d): an LDS double buffer filled through registers with the rows of two k-steps in
//    flight; channel numbers are fetched a step further ahead so the weight loads never wait for them.  Its weight
//    tile has a row stride of 160 elements, which puts the 4 rows of a patch, and the two patches a read instruction's
//    half-wave touches, into disjoint banks.
#include <stdlib.h>

#include "pop_internal.h"

namespace pop {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

constexpr int kDgBM = 256;            // tokens per workgroup tile
constexpr int kDgBN = 128;            // output columns per workgroup tile
constexpr int kDgBK = 64;             // channels per k-step
constexpr int kDgLdA = kDgBK + 8;     // LDS row stride of the Hc tile in elements (144 B: conflict-free 16-byte reads)
constexpr int kDgLdB = kDgBN + 32;    // LDS row stride of the weight tile in elements (320 B)
constexpr int kDgMaxSplit = 8;

__device__ __forceinline__ int dg_xcd_logical_block(int bid, int per_xcd) { return (bid % 8) * per_xcd + bid / 8; }

__global__ __launch_bounds__(512) void down_gemm_bf16_kernel(const uint16_t *__restrict__ w, int d,
                                                             const int *__restrict__ list,
                                                             const int *__restrict__ n_list,
                                                             const uint16_t *__restrict__ hc, int ldh, int T, int n_tt,
                                                             int n_nt, int n_split, int per_xcd,
                                                             float *__restrict__ part, void *__restrict__ y, int y_bf16)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t dg_lds[];
    uint16_t *As = dg_lds;                          // [2][kDgBM * kDgLdA]
    uint16_t *Bs = dg_lds + 2 * kDgBM * kDgLdA;     // [2][kDgBK * kDgLdB]

    const int logical = dg_xcd_logical_block(blockIdx.x, per_xcd);
    if (logical >= n_tt * n_nt * n_split) return;
    // token tiles of one (split, column tile) are neighbours: they share its weight rows in the XCD's L2
    const int ttile = logical % n_tt, ntile = (logical / n_tt) % n_nt, split = logical / (n_tt * n_nt);
    const int t0 = ttile * kDgBM, n0 = ntile * kDgBN;

    const int a = *n_list;
    const int steps_all = (a + kDgBK - 1) / kDgBK, steps_per = (steps_all + n_split - 1) / n_split;
    const int ks0 = min(split * steps_per, steps_all), ks1 = min(ks0 + steps_per, steps_all);

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int wm = wave / 2, wn = wave % 2;

    // staging.  Hc tile: 8 vectors of 16 bytes per row, 64 rows per pass, 4 passes; weight tile: 16 vectors per row,
    // 32 rows per pass, 2 passes
    const int a_row = tid / 8, a_kv = tid % 8;
    const int b_row = tid / 16, b_nv = tid % 16;
    // Every load below is unconditional (addresses clamped into valid memory, the value replaced afterwards where it
    // must not count), so that the loads of two k-steps can be in flight at once: with loads under branches the
    // compiler can only wait for all of them.  Token rows beyond T are clamped and never stored.
    const uint16_t *pa[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) pa[p] = hc + (size_t)min(t0 + a_row + p * 64, T - 1) * ldh;
    const bool n_ok = n0 + b_nv * 8 < d;
    const int n_col = n_ok ? n0 + b_nv * 8 : 0;
    uint4 ra[2][4], rb[2][2];  // two k-steps on their way through registers, as loaded
    uint32_t rb_on[2][2];      // all ones where the weight row exists, else 0
    int chn[2][2], chn_off[2][2];  // channels of this thread's two weight rows, two k-steps, as loaded; -1 where the
                                   // row does not exist, else 0 (kept apart so that nothing touches the loaded value
                                   // before its use a step later)
    auto load_channels = [&](int set, int ks) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int c = ks * kDgBK + b_row + p * 32;
            chn[set][p] = list[min(c, a - 1)];
            chn_off[set][p] = -(int)(ks >= ks1 || c >= a);
        }
    };
    auto load_global = [&](int set, int ks) {
        const int k = min(ks, ks1 - 1) * kDgBK + a_kv * 8;
        const int kc = k < a ? k : 0;
#pragma unroll
        for (int p = 0; p < 4; ++p) ra[set][p] = *reinterpret_cast<const uint4 *>(pa[p] + kc);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int j = chn[set][p] | chn_off[set][p];
            rb[set][p] = *reinterpret_cast<const uint4 *>(w + ((size_t)max(j, 0) * 3 + 2) * d + n_col);
            rb_on[set][p] = (j >= 0 && n_ok) ? 0xffffffffu : 0u;
        }
    };
    // writes the rows of k-step ks, loaded into set `buf`, to LDS buffer `buf`; what lies beyond the a channels or
    // the d columns is cleared here, where the loaded values are first touched
    auto store_lds = [&](int buf, int ks) {
        const int keep = a - (min(ks, ks1 - 1) * kDgBK + a_kv * 8);  // columns of the Hc vector that hold data
        uint32_t keep_bits[4];                                       // 16-bit elements, two per word
#pragma unroll
        for (int q = 0; q < 4; ++q)
            keep_bits[q] = 2 * q >= keep ? 0u : (2 * q + 1 >= keep ? 0xffffu : 0xffffffffu);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint4 v = ra[buf][p];
            *reinterpret_cast<uint4 *>(&As[(buf * kDgBM + a_row + p * 64) * kDgLdA + a_kv * 8]) =
                make_uint4(v.x & keep_bits[0], v.y & keep_bits[1], v.z & keep_bits[2], v.w & keep_bits[3]);
        }
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const uint4 v = rb[buf][p];
            const uint32_t on = rb_on[buf][p];
            *reinterpret_cast<uint4 *>(&Bs[(buf * kDgBK + b_row + p * 32) * kDgLdB + b_nv * 8]) =
                make_uint4(v.x & on, v.y & on, v.z & on, v.w & on);
        }
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;

    // A fragment: row lane % 32 of the token fragment, k = kk + 8 (lane / 32) .. + 7.
    // B fragment, read r (k = kk + 8 (lane / 32) + 4 r .. + 3): this lane points at row (lane % 16) / 4 of that
    // group, columns 16 ((lane / 16) % 2) + 4 (lane % 4) .. + 3 of the fragment, and receives column lane % 32.
    const int a_off = (wm * 64 + lane % 32) * kDgLdA + (lane / 32) * 8;
    const int b_off = ((lane / 32) * 8 + (lane % 16) / 4) * kDgLdB + wn * 64 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);
    auto multiply = [&](int buf) {
        const uint16_t *Ab = As + buf * kDgBM * kDgLdA + a_off;
        const uint16_t *Bb = Bs + buf * kDgBK * kDgLdB + b_off;
#pragma unroll
        for (int kk = 0; kk < kDgBK; kk += 16) {
            bf16x8_t af[2], bf[2];
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const uint16_t *q = Bb + kk * kDgLdB + f * 32;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4_t __attribute__((address_space(3))) *)(q));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4_t __attribute__((address_space(3))) *)(q + 4 * kDgLdB));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bf[f] = __builtin_bit_cast(bf16x8_t, both);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *reinterpret_cast<const bf16x8_t *>(Ab + i * 32 * kDgLdA + kk);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int f = 0; f < 2; ++f)
                    acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[f], acc[i][f], 0, 0, 0);
        }
    };

    // Step ks multiplies LDS buffer (ks - ks0) % 2.  Meanwhile the rows of step ks + 1 are in registers (set of the
    // other parity, requested one step earlier, written to the other buffer after the products), the rows of step
    // ks + 2 are requested into the set this buffer was filled from, and the channel numbers of step ks + 3 are
    // requested ahead of them, so that no wait for an older request also waits for a younger one that is not needed yet.
    const int n_steps = ks1 - ks0;
    if (n_steps > 0) {
        load_channels(0, ks0);
        load_global(0, ks0);
        load_channels(1, ks0 + 1);
        load_global(1, ks0 + 1);
        load_channels(0, ks0 + 2);
        store_lds(0, ks0);
        __syncthreads();
        auto step = [&](int ks, int b) {
            load_channels(b ^ 1, ks + 3);
            load_global(b, ks + 2);
            __builtin_amdgcn_sched_barrier(0);  // (keeps the requests ahead of the products in the instruction stream)
            multiply(b);
            __builtin_amdgcn_sched_barrier(0);
            store_lds(b ^ 1, ks + 1);
            __syncthreads();
        };
        int i = 0;
        for (; i + 1 < n_steps; i += 2) {
            step(ks0 + i, 0);
            step(ks0 + i + 1, 1);
        }
        if (i < n_steps) multiply(0);  // (an odd last step: its rows were stored by the step before)
    }

    // register v of a fragment is token row (v / 4) * 8 + (lane / 32) * 4 + v % 4, column lane % 32
    float *yp = part ? part + (size_t)split * T * d : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int n = n0 + wn * 64 + f * 32 + lane % 32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + wm * 64 + i * 32 + (v / 4) * 8 + (lane / 32) * 4 + v % 4;
                if (t < T && n < d) {
                    const size_t o = (size_t)t * d + n;
                    if (yp) yp[o] = acc[i][f][v];
                    else if (y_bf16) ((uint16_t *)y)[o] = f32_to_bf16(acc[i][f][v]);
                    else ((float *)y)[o] = acc[i][f][v];
                }
            }
        }
}

// The same tile with both operands loaded straight into LDS (global_load_lds) through a ring of three buffers.
// Hc tile: 256 rows x 128 bytes, unpadded, the 16-byte units of row r stored at unit ^ ((r / 2) % 8) (conflict-free
// 16-byte fragment reads).  Weight tile: 64 rows x 256 bytes, unpadded, the units of row k stored at
// unit ^ (4 (k % 4)): the four rows of a transposing read's patch, and the two patches side by side that a half-wave
// touches, then fall into eight different 32-byte bank groups.  Every wave issues the same loads in every k-step (2
// for its weight rows' channel numbers, two steps ahead; 4 + 2 direct loads), so a step waits with an exact count for
// its own rows only.  Nothing is masked: token rows beyond T are pointed at the last token and never stored, list
// positions beyond the a channels are pointed at a row of zeros (zero_row, 256 bytes), which makes it irrelevant what
// the Hc columns beyond a hold, as long as it is finite (the buffer is cleared when it is allocated and only ever
// holds H values).  Needs d % 128 == 0 and ldh >= a rounded up to 64.
constexpr int kDdStages = 3;
constexpr int kDdPerStep = 8;  // vector-memory instructions a wave issues per k-step: 2 channel loads + 6 direct loads

__global__ __launch_bounds__(512) void down_gemm_dma_kernel(const uint16_t *__restrict__ w, int d,
                                                            const int *__restrict__ list,
                                                            const int *__restrict__ n_list,
                                                            const uint16_t *__restrict__ hc, int ldh, int T, int n_tt,
                                                            int n_nt, int n_split, int per_xcd,
                                                            const uint16_t *__restrict__ zero_row,
                                                            float *__restrict__ part, void *__restrict__ y, int y_bf16)
{
    typedef __attribute__((address_space(3))) void lds_t;
    typedef __attribute__((address_space(1))) const void glb_t;
    constexpr int NS = kDdStages;
    constexpr int kATile = kDgBM * kDgBK, kBTile = kDgBK * kDgBN;  // elements per stage
    extern __shared__ __attribute__((aligned(16))) uint16_t dg_lds[];
    uint16_t *As = dg_lds;                 // [NS][256 * 64]
    uint16_t *Bs = dg_lds + NS * kATile;   // [NS][64 * 128]

    const int logical = dg_xcd_logical_block(blockIdx.x, per_xcd);
    if (logical >= n_tt * n_nt * n_split) return;
    const int ttile = logical % n_tt, ntile = (logical / n_tt) % n_nt, split = logical / (n_tt * n_nt);
    const int t0 = ttile * kDgBM, n0 = ntile * kDgBN;

    const int a = *n_list;
    const int steps_all = (a + kDgBK - 1) / kDgBK, steps_per = (steps_all + n_split - 1) / n_split;
    const int ks0 = min(split * steps_per, steps_all), ks1 = min(ks0 + steps_per, steps_all);
    const int n_steps = ks1 - ks0;

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave / 2, wn = wave % 2;

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;

    if (n_steps > 0) {
        // direct loads.  Hc: pass p of wave w covers rows 64 p + 8 w + lane / 8, this lane the unit that belongs at
        // position lane % 8 of its row.  Weights: pass p covers rows 32 p + 4 w + lane / 16, position lane % 16.
        const int a_row = wave * 8 + lane / 8;
        const int a_src = ((lane % 8) ^ ((a_row / 2) % 8)) * 8;   // (passes are 64 rows apart: same swizzle term)
        const uint16_t *pa[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) pa[p] = hc + (size_t)min(t0 + a_row + p * 64, T - 1) * ldh + a_src;
        const int b_row = wave * 4 + lane / 16;
        const int b_src = n0 + ((lane % 16) ^ (4 * (b_row % 4))) * 8;  // (passes are 32 rows apart: same swizzle term)
        // Channel numbers of this lane's two weight rows, for three k-steps (set = step % 3).  They are loaded with
        // inline assembly, two steps before the direct loads that need them: the compiler does not see these loads, so
        // it adds no waits of its own for them (across the loop's back edge those come out as waits for everything);
        // the step's one explicit wait covers them, and passes the registers through so that no use moves above it.
        int chn[3][2];
        auto load_channels = [&](int set, int ks) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int *src = list + min(min(ks, ks1 - 1) * kDgBK + b_row + p * 32, a - 1);
                asm volatile("global_load_dword %0, %1, off" : "=v"(chn[set][p]) : "v"(src) : "memory");
            }
        };
        auto dma_load = [&](int buf, int set, int ks) {
            const int kc = min(ks, ks1 - 1);
#pragma unroll
            for (int p = 0; p < 4; ++p)
                __builtin_amdgcn_global_load_lds((glb_t *)(pa[p] + kc * kDgBK),
                                                 (lds_t *)(As + buf * kATile + (p * 64 + wave_u * 8) * kDgBK), 16, 0, 0);
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                // (selected with a mask: a conditional would put the load under a branch and make its wait inexact)
                const uintptr_t live = -(uintptr_t)(ks < ks1 && ks * kDgBK + b_row + p * 32 < a);
                const uintptr_t p_row = (uintptr_t)(w + ((size_t)chn[set][p] * 3 + 2) * d + b_src);
                const uintptr_t p_zero = (uintptr_t)(zero_row + (lane % 16) * 8);
                const uint16_t *row = (const uint16_t *)(p_zero ^ ((p_row ^ p_zero) & live));
                __builtin_amdgcn_global_load_lds((glb_t *)row,
                                                 (lds_t *)(Bs + buf * kBTile + (p * 32 + wave_u * 4) * kDgBN), 16, 0, 0);
            }
        };
        // fragment addresses.  A: row lane % 32 of the token fragment, unit kk / 8 + lane / 32 under the row's swizzle.
        // B, read r: this lane points at row kk + 8 (lane / 32) + 4 r + (lane % 16) / 4, columns
        // 16 ((lane / 16) % 2) + 4 (lane % 4) .. + 3 of the fragment, and receives column lane % 32.
        const int arow = wm * 64 + lane % 32, a_sw = (arow / 2) % 8;  // (fragments are 32 rows apart: same term)
        const int b_k = (lane / 32) * 8 + (lane % 16) / 4, b_sw = 4 * (b_k % 4);
        const int b_col = wn * 64 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);
        // The fragment reads are issued as inline assembly: as an intrinsic the compiler takes the transposing read to
        // alias the direct loads in flight and waits for all of those first.  It therefore does not count these reads
        // either; the explicit waits below do: the reads of k-slice q + 1 are issued before the products of slice q,
        // which wait for all reads but those six.
        auto tr_read = [&](s16x4_t &v, const uint16_t *q) {
            asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"((uint32_t)(uintptr_t)q));
        };
        auto a_read = [&](bf16x8_t &v, const uint16_t *q) {
            asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"((uint32_t)(uintptr_t)q));
        };
        auto multiply = [&](int buf) {
            const uint16_t *Ab = As + buf * kATile + arow * kDgBK;
            const uint16_t *Bb = Bs + buf * kBTile + b_k * kDgBN;
            bf16x8_t af[2][2];
            s16x4_t lo[2][2], hi[2][2];
            auto fetch = [&](int q, int set) {
#pragma unroll
                for (int f = 0; f < 2; ++f) {
                    const int col = b_col + f * 32;
                    const uint16_t *p = Bb + q * 16 * kDgBN + (((col / 8) ^ b_sw) * 8) + col % 8;
                    tr_read(lo[set][f], p);
                    tr_read(hi[set][f], p + 4 * kDgBN);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    a_read(af[set][i], Ab + i * 32 * kDgBK + (((q * 2 + lane / 32) ^ a_sw) * 8));
            };
            fetch(0, 0);
#pragma unroll
            for (int q = 0; q < kDgBK / 16; ++q) {
                const int c = q & 1;
                if (q + 1 < kDgBK / 16) {
                    fetch(q + 1, c ^ 1);
                    asm volatile("s_waitcnt lgkmcnt(6)"
                                 : "+v"(lo[c][0]), "+v"(hi[c][0]), "+v"(lo[c][1]), "+v"(hi[c][1]), "+v"(af[c][0]), "+v"(af[c][1])
                                 :
                                 : "memory");
                } else {
                    asm volatile("s_waitcnt lgkmcnt(0)"
                                 : "+v"(lo[c][0]), "+v"(hi[c][0]), "+v"(lo[c][1]), "+v"(hi[c][1]), "+v"(af[c][0]), "+v"(af[c][1])
                                 :
                                 : "memory");
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int f = 0; f < 2; ++f) {
                        const bf16x8_t bf = __builtin_bit_cast(
                            bf16x8_t, __builtin_shufflevector(lo[c][f], hi[c][f], 0, 1, 2, 3, 4, 5, 6, 7));
                        acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], bf, acc[i][f], 0, 0, 0);
                    }
            }
        };

        // Step ks0 + i multiplies buffer i % 3.  Per step: wait until this wave's direct loads of the step have landed
        // (all but the kDdPerStep instructions of the step after it), meet the other waves (now everybody's have, and
        // everybody is done reading the buffer of the step before), request the channel numbers of the step four
        // ahead and the rows of the step two ahead (into that buffer; its channel numbers were requested before the
        // rows of this step, so they have arrived too), multiply.  Steps beyond the last are requested as rows of
        // zeros (weights) and again from the last step (Hc), so the count holds.
        static_assert((NS - 2) * kDdPerStep == 8, "the wait below allows the 8 instructions of the next step");
#define POP_DD_CHN "+v"(chn[0][0]), "+v"(chn[0][1]), "+v"(chn[1][0]), "+v"(chn[1][1]), "+v"(chn[2][0]), "+v"(chn[2][1])
        load_channels(0, ks0);
        load_channels(1, ks0 + 1);
        load_channels(2, ks0 + 2);
        asm volatile("s_waitcnt vmcnt(0)" : POP_DD_CHN : : "memory");
        dma_load(0, 0, ks0);
        dma_load(1, 1, ks0 + 1);
        load_channels(0, ks0 + 3);
        // step i (buffer and channel set b = i % 3, fixed by unrolling three steps per trip)
        auto step = [&](int i, int b) {
            asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" : POP_DD_CHN : : "memory");  // (no fence: it would wait for all)
            load_channels((b + 1) % 3, ks0 + i + 4);
            dma_load((b + 2) % 3, (b + 2) % 3, ks0 + i + 2);
            __builtin_amdgcn_sched_barrier(0);
            multiply(b);
        };
        int i = 0;
        for (; i + 3 <= n_steps; i += 3) {
            step(i, 0);
            step(i + 1, 1);
            step(i + 2, 2);
        }
        if (i < n_steps) step(i, 0);
        if (i + 1 < n_steps) step(i + 1, 1);
        // the surplus requests, before the LDS is given up; the channel registers are operands so that they stay
        // allocated until the loads into them have landed (the last ones are never used)
        asm volatile("s_waitcnt vmcnt(0)" : POP_DD_CHN : : "memory");
#undef POP_DD_CHN
    }

    // register v of a fragment is token row (v / 4) * 8 + (lane / 32) * 4 + v % 4, column lane % 32
    float *yp = part ? part + (size_t)split * T * d : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int n = n0 + wn * 64 + f * 32 + lane % 32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + wm * 64 + i * 32 + (v / 4) * 8 + (lane / 32) * 4 + v % 4;
                if (t < T && n < d) {
                    const size_t o = (size_t)t * d + n;
                    if (yp) yp[o] = acc[i][f][v];
                    else if (y_bf16) ((uint16_t *)y)[o] = f32_to_bf16(acc[i][f][v]);
                    else ((float *)y)[o] = acc[i][f][v];
                }
            }
        }
}

// y = sum over the splits, in split order, of part[split]; n4 = T * d / 4 vectors.
__global__ __launch_bounds__(256) void down_gemm_reduce_kernel(const float4 *__restrict__ part, int n_split, size_t n4,
                                                               void *__restrict__ y, int y_bf16)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    float4 s = part[i];
    for (int q = 1; q < n_split; ++q) {
        const float4 v = part[(size_t)q * n4 + i];
        s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
    }
    if (y_bf16) {
        uint2 o;
        o.x = (uint32_t)f32_to_bf16(s.x) | ((uint32_t)f32_to_bf16(s.y) << 16);
        o.y = (uint32_t)f32_to_bf16(s.z) | ((uint32_t)f32_to_bf16(s.w) << 16);
        ((uint2 *)y)[i] = o;
    } else {
        ((float4 *)y)[i] = s;
    }
}

// Ranges the contraction is split into so that the tiles fill the compute units.
int down_gemm_splits(int T, int d, int n_cu)
{
    const int tiles = ((T + kDgBM - 1) / kDgBM) * ((d + kDgBN - 1) / kDgBN);
    int n_split = n_cu / tiles;
    if (n_split < 1) n_split = 1;
    if (n_split > kDgMaxSplit) n_split = kDgMaxSplit;
    return n_split;
}

// bf16 only; d % 8 == 0, ldh % 8 == 0.  part: float32 [n_split][T][d], needed when n_split > 1.  zero_row: 256 bytes
// of zeros (optional); with it, d % 128 == 0 and ldh % 64 == 0 the direct-load kernel runs (POP_DG_DMA=0 keeps the
// register-staged one, for comparison), which reads Hc columns up to the list length rounded up to 64.
hipError_t launch_down_gemm_bf16(const void *w, int d, const int *list, const int *n_list, const uint16_t *hc, int ldh,
                                 int T, int n_split, float *part, void *y, int y_bf16, hipStream_t s,
                                 const uint16_t *zero_row)
{
    static const int use_dma = getenv("POP_DG_DMA") ? atoi(getenv("POP_DG_DMA")) : 1;
    const int n_tt = (T + kDgBM - 1) / kDgBM, n_nt = (d + kDgBN - 1) / kDgBN;
    const int total = n_tt * n_nt * n_split, per_xcd = (total + 7) / 8;
    hipError_t e;
    if (use_dma && zero_row && d % kDgBN == 0 && ldh % kDgBK == 0) {
        const size_t lds = (size_t)kDdStages * (kDgBM * kDgBK + kDgBK * kDgBN) * sizeof(uint16_t);
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&down_gemm_dma_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(down_gemm_dma_kernel, dim3(per_xcd * 8), dim3(512), lds, s, (const uint16_t *)w, d, list,
                           n_list, hc, ldh, T, n_tt, n_nt, n_split, per_xcd, zero_row, n_split > 1 ? part : nullptr, y,
                           y_bf16);
    } else {
        const size_t lds = (size_t)2 * (kDgBM * kDgLdA + kDgBK * kDgLdB) * sizeof(uint16_t);
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&down_gemm_bf16_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(down_gemm_bf16_kernel, dim3(per_xcd * 8), dim3(512), lds, s, (const uint16_t *)w, d, list,
                           n_list, hc, ldh, T, n_tt, n_nt, n_split, per_xcd, n_split > 1 ? part : nullptr, y, y_bf16);
    }
    e = hipGetLastError();
    if (e != hipSuccess || n_split <= 1) return e;
    const size_t n4 = (size_t)T * d / 4;
    hipLaunchKernelGGL(down_gemm_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (const float4 *)part,
                       n_split, n4, y, y_bf16);
    return hipGetLastError();
}

}  // namespace pop
