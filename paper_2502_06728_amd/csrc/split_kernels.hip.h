// Lane per chunk, wavefront per coefficient class: the compress half for chunk sizes above 64.
//
// A chunk of more than 64 elements does not fit one lane's registers at two wavefronts per
// SIMD.  Splitting it between two lanes of ONE wavefront makes the lanes run different
// half-size transforms (a DCT-II and a DCT-IV) one after the other.  Here the split is between
// the W wavefronts of a workgroup instead: the workgroup owns a tile of 64 chunks in LDS
// (row = chunk), lane t of EVERY wavefront works on chunk t, and wavefront w computes one class
// of the chunk's coefficients, S/W of them, in its lanes' registers.  Every wavefront runs
// straight-line code with no divergence, and the classes meet in LDS at workgroup barriers.
//
//   W = 2 (chunk 96, 128), first level of the DCT-II recursion of fast_dct.hip.h:
//     class 0: u_n = x_n + x_{S-1-n}, coefficients 2m   = dct2_{S/2}(u)
//     class 1: w_n = x_n - x_{S-1-n}, coefficients 2m+1 = dct4_{S/2}(w)
//   W = 4 (chunk 192, 256), two levels, Q = S/4:
//     class 0: coefficients 4m   = dct2_Q(u_n + u_{S/2-1-n})
//     class 1: coefficients 4m+2 = dct4_Q(u_n - u_{S/2-1-n})
//     class 2, 3: the DCT-IV of w (length S/2) by plane rotations into two DCT-IIs of length
//              Q, A (class 2) and B (class 3); after an exchange through LDS class 2 holds the
//              coefficients 4m+1 = A_m + B_{Q-m} and class 3 the coefficients
//              4m+3 = A_{m+1} - B_{Q-1-m}.
// The inverse runs the same splits backwards (DCT-III / DCT-IV).
//
// Selection (top-k, any k at run time): every lane sorts the magnitudes of its S/W coefficients
// with a sorting network; the sorted lists of a chunk meet in the chunk's LDS row.  For W = 4
// the lists of classes (0,1) and (2,3) are first merged into two sorted lists of 128 (one
// bitonic half-cleaner across the two wavefronts, then a bitonic merge network per lane).  The
// k-th largest of the union of two sorted lists follows from a binary search over how many of
// the k come from the first list.  A tie at the threshold sends the chunk through the
// whole-wavefront pass that keeps the lowest indices among the equals.
//
// Emission: every class knows the other classes' kept sets as bit masks (exchanged through
// LDS), so a lane can tell the payload position of each of its kept coefficients: its rank
// among all kept coefficients of the chunk with a smaller index.  Values and indices are staged
// in the chunk's row and leave with coalesced stores.
#pragma once

#include "fast_dct.hip.h"
#include "generic_kernels.hip.h"
#include "mfma_kernels.hip.h"
#include "sort_network.hip.h"

namespace deto {

template <int S, int W>
struct SplitGeom {
    static_assert(W == 2 || W == 4, "two or four coefficient classes");
    static_assert(S % (4 * W) == 0, "16-byte pieces per class");
    static constexpr int Q = S / W;                 // coefficients per lane
    static constexpr int kRow = S + 4;              // floats per LDS row (16 B of padding)
    static constexpr int kTile = kWave * kRow;
    static constexpr int kThreads = kWave * W;
    static constexpr int NW = (Q + 31) / 32;        // mask words per lane
    // payload staging inside a chunk's row: values at row[pos], indices at row[kIdx0 + pos]
    // (k <= S/2); what a lane drops goes to a dump slot of its own: past the tile in general,
    // inside its row when k <= kRowDumpMaxK leaves room there (value at row[kRowDump + a], its
    // index kIdx0 further on in the row's padding, row[S + a]; a = lane / 16 spreads the 64
    // lanes of a wavefront over the 64 banks: the row stride is 4 banks.  The classes of a
    // chunk share the slot: nobody reads it)
    static constexpr int kIdx0 = S / 2 + 4;
    static constexpr int kRowDump = S / 2 - 4;
    static constexpr int kRowDumpMaxK = S / 2 - 4;
    static constexpr int kBufFloats = kTile + kThreads + kIdx0;
};

// index of coefficient m of class w: W*m + split_off(w)
template <int W>
__device__ __forceinline__ int split_off(int w) {
    if constexpr (W == 2) return w;
    else return ((w & 1) << 1) | (w >> 1);          // 0, 2, 1, 3
}

// k-th largest of the union of two descending lists of length L in LDS: i of the k largest
// come from list 0 and k - i from list 1, i being the smallest count for which list0[i] (the
// first one left out) does not exceed list1[k-i-1] (the last one taken).
template <int L>
__device__ __forceinline__ uint32_t kth_of_two_lists(const uint32_t* l0, const uint32_t* l1,
                                                     int k) {
    int lo = k > L ? k - L : 0, hi = k < L ? k : L;
    constexpr int kSteps = L <= 63 ? 6 : (L <= 127 ? 7 : 8);   // ceil(log2(L + 1))
#pragma unroll
    for (int it = 0; it < kSteps; ++it) {
        const bool open = lo < hi;
        const int mid = (lo + hi) >> 1;
        const uint32_t x0 = l0[open ? mid : 0];
        const uint32_t x1 = l1[open ? k - mid - 1 : 0];
        if (open) {
            if (x0 > x1) lo = mid + 1;
            else hi = mid;
        }
    }
    const int n0 = lo, n1 = k - lo;
    const uint32_t t0 = l0[n0 > 0 ? n0 - 1 : 0], t1 = l1[n1 > 0 ? n1 - 1 : 0];
    return min(n0 > 0 ? t0 : 0xFFFFFFFFu, n1 > 0 ? t1 : 0xFFFFFFFFu);
}

// 2*word + (mag >= thr): a compare into the carry and an add with carry
__device__ __forceinline__ uint32_t push_if_at_least(uint32_t word, uint32_t mag, uint32_t thr) {
    asm("v_cmp_ge_u32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
        : "+v"(word)
        : "v"(mag), "v"(thr)
        : "vcc");
    return word;
}

template <int Q>
__device__ __forceinline__ void regs_to_lds(float* dst, const float (&v)[Q]) {
#pragma unroll
    for (int q = 0; q < Q / 4; ++q)
        *reinterpret_cast<float4*>(dst + 4 * q) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}

template <int Q>
__device__ __forceinline__ void lds_to_regs(const float* src, float (&v)[Q]) {
#pragma unroll
    for (int q = 0; q < Q / 4; ++q) {
        const float4 t = *reinterpret_cast<const float4*>(src + 4 * q);
        v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
    }
}

// src[Q-1-i] for i < Q (a list read back to front)
template <int Q>
__device__ __forceinline__ void lds_to_regs_reversed(const float* src, float (&v)[Q]) {
#pragma unroll
    for (int q = 0; q < Q / 4; ++q) {
        const float4 t = *reinterpret_cast<const float4*>(src + Q - 4 - 4 * q);
        v[4 * q] = t.w; v[4 * q + 1] = t.z; v[4 * q + 2] = t.y; v[4 * q + 3] = t.x;
    }
}

// ---- forward: the lane's class of coefficients (unscaled) from the chunk's row
template <int S, int W>
__device__ __forceinline__ void split_forward_local(const float* __restrict__ row, int w,
                                                    float (&c)[S / W]) {
    constexpr int Q = S / W;
    if constexpr (W == 2) {
        const float sgn = w ? -1.0f : 1.0f;
#pragma unroll
        for (int q = 0; q < Q / 4; ++q) {
            const float4 a = *reinterpret_cast<const float4*>(row + 4 * q);
            const float4 b = *reinterpret_cast<const float4*>(row + S - 4 - 4 * q);
            c[4 * q] = fmaf(sgn, b.w, a.x);
            c[4 * q + 1] = fmaf(sgn, b.z, a.y);
            c[4 * q + 2] = fmaf(sgn, b.y, a.z);
            c[4 * q + 3] = fmaf(sgn, b.x, a.w);
        }
        if (w == 0) FastDct<Q>::dct2(c);
        else FastDct<Q>::dct4(c);
    } else {
        constexpr int H = S / 2;
        // four elements at a time: x[n], x[S-1-n], x[H-1-n], x[H+n] for n = 4q .. 4q+3
        static_for<0, Q / 4>([&](auto q) {
            const float4 f0 = *reinterpret_cast<const float4*>(row + 4 * q);
            const float4 r1 = *reinterpret_cast<const float4*>(row + S - 4 - 4 * q);
            const float4 r2 = *reinterpret_cast<const float4*>(row + H - 4 - 4 * q);
            const float4 f3 = *reinterpret_cast<const float4*>(row + H + 4 * q);
            const float x0[4] = {f0.x, f0.y, f0.z, f0.w};
            const float x1[4] = {r1.w, r1.z, r1.y, r1.x};
            const float x2[4] = {r2.w, r2.z, r2.y, r2.x};
            const float x3[4] = {f3.x, f3.y, f3.z, f3.w};
            static_for<0, 4>([&](auto i) {
                constexpr int j = 4 * q + i;
                if (w < 2) {
                    const float sgn = w ? -1.0f : 1.0f;
                    c[j] = fmaf(sgn, x2[i] + x3[i], x0[i] + x1[i]);
                } else {
                    // rotations of the DCT-IV of w (length H): pair (w_j, w_{H-1-j})
                    constexpr float cs = Rot<H, j>::c, sn = Rot<H, j>::s;
                    const float wj = x0[i] - x1[i], wr = x2[i] - x3[i];
                    const float av = fmaf(wj, cs, wr * sn);
                    const float bv = fmaf(wr, cs, -(wj * sn));
                    c[j] = (w == 2) ? av : ((j % 2) ? -bv : bv);
                }
            });
        });
        if (w == 1) FastDct<Q>::dct4(c);
        else FastDct<Q>::dct2(c);
    }
}

// W = 4: classes 2 and 3 hold A and B; after this class 2 holds the coefficients 4m+1 and
// class 3 the coefficients 4m+3.  The tile rows must be free; contains workgroup barriers,
// every wavefront calls it.
template <int S>
__device__ __forceinline__ void split_forward_exchange(float* __restrict__ row, int w,
                                                       float (&c)[S / 4]) {
    constexpr int Q = S / 4;
    if (w >= 2) regs_to_lds<Q>(row + (w - 2) * Q, c);
    __syncthreads();
    if (w == 2) {
        // c[l] = A[l] + B[Q-l] for l >= 1
        float br[Q];
        lds_to_regs_reversed<Q>(row + Q, br);        // br[i] = B[Q-1-i]
        static_for<1, Q>([&](auto l) { c[l] += br[l - 1]; });
    } else if (w == 3) {
        // c[l] = A[l+1] - B[Q-1-l] for l < Q-1, c[Q-1] = -B[0]
        float a[Q], d[Q];
        lds_to_regs<Q>(row, a);
        static_for<0, Q - 1>([&](auto l) { d[l] = a[l + 1] - c[Q - 1 - l]; });
        d[Q - 1] = -c[0];
#pragma unroll
        for (int l = 0; l < Q; ++l) c[l] = d[l];
    }
    __syncthreads();
}

// ---- inverse: the classes' scaled coefficients back into the rows as [E | O] (W = 2) or
// [E (128) | O even (64) | O odd (64)] (W = 4), ready for split_output.  Contains workgroup
// barriers; the rows must be free on entry.
template <int S, int W>
__device__ __forceinline__ void split_inverse_to_rows(float* __restrict__ row, int w,
                                                      float (&c)[S / W]) {
    constexpr int Q = S / W;
    if constexpr (W == 2) {
        if (w == 0) FastDct<Q>::dct3(c);
        else FastDct<Q>::dct4(c);
        regs_to_lds<Q>(row + w * Q, c);
        __syncthreads();
    } else {
        // classes 2 and 3 exchange their coefficients: v[j] = coefficient 2j+1 of the chunk,
        // v[2l] = class 2's c[l], v[2l+1] = class 3's c[l]
        constexpr int H = S / 2;
        if (w >= 2) regs_to_lds<Q>(row + H + (w - 2) * Q, c);
        __syncthreads();
        if (w == 0) {
            FastDct<Q>::dct3(c);
        } else if (w == 1) {
            FastDct<Q>::dct4(c);
        } else {
            // the Q rotation pairs, eight at a time: four entries of the other class from the
            // front and four from the back
            static_assert(Q % 8 == 0, "whole blocks of eight pairs");
            const float* other = row + H + (3 - w) * Q;
            float r[Q];
            static_for<0, Q / 8>([&](auto q) {
                const float4 fo = *reinterpret_cast<const float4*>(other + 4 * q);
                const float4 ro = *reinterpret_cast<const float4*>(other + Q - 4 - 4 * q);
                const float o[4] = {fo.x, fo.y, fo.z, fo.w};          // other[l]
                const float orv[4] = {ro.w, ro.z, ro.y, ro.x};        // other[Q-1-l]
                static_for<0, 8>([&](auto i) {
                    constexpr int j = 8 * q + i;
                    constexpr int l = j / 2, li = l - 4 * q;
                    constexpr float cs = Rot<H, j>::c, sn = Rot<H, j>::s;
                    // pair (v[j], v[H-1-j]): j even: (c2[l], c3[Q-1-l]); j odd: (c3[l], c2[Q-1-l])
                    float pj, qj;
                    if (w == 2) {
                        pj = (j % 2) ? o[li] : c[l];
                        qj = (j % 2) ? c[Q - 1 - l] : orv[li];
                    } else {
                        pj = (j % 2) ? c[l] : o[li];
                        qj = (j % 2) ? orv[li] : c[Q - 1 - l];
                    }
                    const float av = fmaf(pj, cs, qj * sn);
                    const float bv = fmaf(qj, cs, -(pj * sn));
                    r[j] = (w == 2) ? av : ((j % 2) ? -bv : bv);
                });
            });
            FastDct<Q>::dct2(r);
#pragma unroll
            for (int j = 0; j < Q; ++j) c[j] = r[j];
        }
        __syncthreads();
        // EE | EO | A | B
        regs_to_lds<Q>(row + w * Q, c);
        __syncthreads();
        float f[Q];
        if (w == 0) {
            float eo[Q];
            lds_to_regs<Q>(row + Q, eo);
#pragma unroll
            for (int i = 0; i < Q; ++i) f[i] = c[i] + eo[i];            // E[i]
        } else if (w == 1) {
            float ee[Q];
            lds_to_regs_reversed<Q>(row, ee);                            // ee[m] = EE[63-m]
            // E[64+m] = E[127-(63-m)] = EE[63-m] - EO[63-m]
#pragma unroll
            for (int m = 0; m < Q; ++m) f[m] = ee[m] - c[Q - 1 - m];
        } else if (w == 2) {
            float br[Q];
            lds_to_regs_reversed<Q>(row + 3 * Q, br);                    // br[i] = B[63-i]
            f[0] = c[0];
            static_for<1, Q>([&](auto l) { f[l] = c[l] + br[l - 1]; });   // O[2l]
        } else {
            float a[Q];
            lds_to_regs<Q>(row + 2 * Q, a);
            static_for<0, Q - 1>([&](auto l) { f[l] = a[l + 1] - c[Q - 1 - l]; });   // O[2l+1]
            f[Q - 1] = -c[0];
        }
        __syncthreads();
        regs_to_lds<Q>(row + w * Q, f);
        __syncthreads();
    }
}

// four consecutive elements col .. col+3 of the chunk whose row was left by
// split_inverse_to_rows
template <int S, int W>
__device__ __forceinline__ float4 split_output(const float* __restrict__ row, int col) {
    constexpr int H = S / 2;
    const bool upper = col >= H;
    const int n0 = upper ? S - 4 - col : col;     // elements col+i mirror n0+3-i when upper
    const float4 e = *reinterpret_cast<const float4*>(row + n0);
    float4 o;
    if constexpr (W == 2) {
        o = *reinterpret_cast<const float4*>(row + H + n0);
    } else {
        const float2 oe = *reinterpret_cast<const float2*>(row + H + n0 / 2);
        const float2 oo = *reinterpret_cast<const float2*>(row + H + H / 2 + n0 / 2);
        o = make_float4(oe.x, oo.x, oe.y, oo.y);
    }
    if (!upper) return make_float4(e.x + o.x, e.y + o.y, e.z + o.z, e.w + o.w);
    return make_float4(e.w - o.w, e.z - o.z, e.y - o.y, e.x - o.x);
}

// Compress half (top-k, DCT domain, fp32 values + int32 indices, k <= S/2) on full tiles of 64
// chunks; the chunks past the last full tile form one partial tile (one more workgroup).
// TOP > 0: for launches with k <= TOP (see the selection step).
// Occupancy: the workgroups of a CU are each in one phase at a time (barriers), so the number
// of workgroups per CU is what overlaps memory phases with arithmetic.  Chunk 192 with the
// partial sort fits three (168 registers, 52 KB of LDS with the dump slots inside the rows);
// chunk 256 two (a 64-row tile alone is 65 KB); chunk 96 / 128 four to six of two wavefronts.
template <int S, int W, bool GRAD_BF16, int TOP = 0>
__global__ __launch_bounds__(kWave * W)
__attribute__((amdgpu_waves_per_eu((S == 192 && TOP > 0) ? 3 : 2))) void compress_split(
    KParams p, int64_t tiles, int64_t n, int64_t n_chunks, const void* __restrict__ grad,
    float* __restrict__ mom, int32_t* __restrict__ idx_out, float* __restrict__ val_out,
    float* __restrict__ coeff_dbg) {
    using G = SplitGeom<S, W>;
    constexpr int Q = G::Q, kRow = G::kRow, NW = G::NW, kThreads = G::kThreads;
    constexpr int kIdx0 = G::kIdx0, kTile = G::kTile;
    // a launch with the partial sort has k <= TOP: the dump slots fit into the rows
    constexpr bool kRowDumps = TOP > 0 && TOP <= G::kRowDumpMaxK;
    __shared__ __attribute__((aligned(16))) float buf[kRowDumps ? G::kTile : G::kBufFloats];
    __shared__ uint32_t s_mask[kWave][W][NW];    // kept sets: chunk, class, word
    __shared__ uint8_t s_cnt[kWave][W];          // kept per class (at most Q <= 64)
    __shared__ unsigned long long s_tie;         // chunks of the tile that took the tie pass

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = p.k;

    // Workgroups [0, tiles): full tiles.  The chunks left over (fewer than 64, the last of them
    // possibly ragged: the shard need not end on a chunk boundary) form ONE partial tile: its
    // first `live` rows are chunks, the other lanes idle; positions past the end of the shard
    // read as zero and are never written.
    const int64_t tile = blockIdx.x;
    const bool partial = tile >= tiles;    // (a partial tile can have 64 rows, the last ragged)
    const int live = partial ? static_cast<int>(n_chunks - tiles * kWave) : kWave;
    const bool alive = lane < live;
    const int64_t base = tile * static_cast<int64_t>(kWave * S);
    const int64_t chunk0 = tile * kWave;
    float* row = &buf[lane * kRow];
    if (tid == 0) s_tie = 0ull;

    // ---- m1 = beta*m + g for the tile's contiguous elements, coalesced, into the rows (the
    // rows past a partial tile's chunks become zero)
    {
        constexpr int kIt = Q / 4;               // 16-byte pieces per thread
        auto fold_piece = [&](int e4) {
            const int r = e4 / S, col = e4 - r * S;
            const float4 m = ld_f4<false>(mom + base + e4);
            float4 g;
            if constexpr (GRAD_BF16) {
                const uint2 gb = ld_u2<false>(static_cast<const uint16_t*>(grad) + base + e4);
                g = make_float4(__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xFFFF0000u),
                                __uint_as_float(gb.y << 16), __uint_as_float(gb.y & 0xFFFF0000u));
            } else {
                g = ld_f4<false>(static_cast<const float*>(grad) + base + e4);
            }
            *reinterpret_cast<float4*>(&buf[r * kRow + col]) =
                make_float4(fmaf(p.beta, m.x, g.x), fmaf(p.beta, m.y, g.y),
                            fmaf(p.beta, m.z, g.z), fmaf(p.beta, m.w, g.w));
        };
        if (!partial) {
#pragma unroll
            for (int it = 0; it < kIt; ++it) fold_piece(4 * (tid + kThreads * it));
        } else {
            for (int it = 0; it < kIt; ++it) {
                const int e4 = 4 * (tid + kThreads * it);
                const int64_t i0 = base + e4;
                if (i0 + 3 < n) {
                    fold_piece(e4);
                } else {
                    // the piece that straddles the end of the shard, and everything past it
                    const int r = e4 / S, col = e4 - r * S;
                    float x[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        x[j] = 0.0f;
                        if (i0 + j < n) {
                            const float g = GRAD_BF16
                                ? bf16_to_f32(static_cast<const uint16_t*>(grad)[i0 + j])
                                : static_cast<const float*>(grad)[i0 + j];
                            x[j] = fmaf(p.beta, mom[i0 + j], g);
                        }
                    }
                    *reinterpret_cast<float4*>(&buf[r * kRow + col]) =
                        make_float4(x[0], x[1], x[2], x[3]);
                }
            }
        }
    }
    __syncthreads();

    // ---- the lane's coefficients c[m] = coefficient W*m + off of chunk `lane`
    const int off = split_off<W>(w);
    float c[Q];
    split_forward_local<S, W>(row, w, c);
    __syncthreads();                              // every class has read the chunk: rows free
    if constexpr (W == 4) split_forward_exchange<S>(row, w, c);
    c[0] *= (w == 0) ? p.alpha0 : p.alpha;
#pragma unroll
    for (int m = 1; m < Q; ++m) c[m] *= p.alpha;
    if (coeff_dbg && alive) {
        float* dbg = coeff_dbg + (chunk0 + lane) * S + off;
#pragma unroll
        for (int m = 0; m < Q; ++m) dbg[W * m] = c[m];
    }

    // ---- k-th largest magnitude T of the chunk
    uint32_t T;
    {
        // (the magnitudes are formed again when the kept sets are marked: keeping these
        // copies alive across the sort would cost Q registers)
        uint32_t a[Q];
#pragma unroll
        for (int m = 0; m < Q; ++m) {
            a[m] = __float_as_uint(c[m]) & 0x7FFFFFFFu;
            asm volatile("" : "+v"(a[m]));
        }
        uint32_t* lists = reinterpret_cast<uint32_t*>(row);
        auto publish = [&]() {
#pragma unroll
            for (int q = 0; q < Q / 4; ++q)
                *reinterpret_cast<uint4*>(lists + w * Q + 4 * q) =
                    make_uint4(a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]);
        };
        // each class contributes at most k of the k largest: a launch with k <= TOP sorts out
        // only every lane's largest TOP (TOP = 0: the full sort)
        if constexpr (TOP > 0) sort_top_desc<Q, TOP>(a);
        else sort_desc<Q>(a);
        publish();
        __syncthreads();
        if constexpr (W == 4 && TOP > 0) {
            // only the TOP largest of each class are in the lists (k <= TOP): the TOP largest
            // of a pair of classes are the maxima of one list against the mirror image of the
            // other, a bitonic sequence that the even class of the pair sorts; the odd class
            // waits.  The pair's merged list has TOP entries.
            uint32_t x[TOP];
            if ((w & 1) == 0) {
                const uint32_t* mine = lists + w * Q;
                const uint32_t* partner = lists + (w + 1) * Q;
                static_for<0, TOP / 4>([&](auto q) {
                    const uint4 m4 = *reinterpret_cast<const uint4*>(mine + 4 * q);
                    const uint4 t = *reinterpret_cast<const uint4*>(partner + TOP - 4 - 4 * q);
                    x[4 * q] = max(m4.x, t.w);
                    x[4 * q + 1] = max(m4.y, t.z);
                    x[4 * q + 2] = max(m4.z, t.y);
                    x[4 * q + 3] = max(m4.w, t.x);
                });
                bitonic_merge_desc<TOP>(x);
            }
            __syncthreads();
            if ((w & 1) == 0) {
                uint32_t* merged = lists + (w >> 1) * 2 * Q;
#pragma unroll
                for (int q = 0; q < TOP / 4; ++q)
                    *reinterpret_cast<uint4*>(merged + 4 * q) =
                        make_uint4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
            }
            __syncthreads();
            T = kth_of_two_lists<TOP>(lists, lists + 2 * Q, k);
        } else if constexpr (W == 4) {
            // classes (0,1) and (2,3): the larger half of the two lists' union to the even
            // class, the smaller half to the odd one; each half is bitonic and is sorted in
            // place.  Lists are padded with zeros (the smallest magnitude) to a power of two
            // QP; the even class ends up with the QP largest, the odd one with the other
            // 2Q - QP followed by padding, so the pair's merged list has 2Q entries again.
            constexpr int QP = SortNet<Q>::P;
            const uint32_t* partner = lists + (w ^ 1) * Q;
            uint32_t x[QP];
            static_for<0, QP / 4>([&](auto q) {
                constexpr int j0 = QP - 4 - 4 * q;               // partner's entries j0 .. j0+3
                uint4 t = make_uint4(0u, 0u, 0u, 0u);
                if constexpr (j0 < Q) t = *reinterpret_cast<const uint4*>(partner + j0);
                const uint32_t theirs[4] = {t.w, t.z, t.y, t.x};  // partner[QP-1-i], i = 4q ..
                uint4 m4 = make_uint4(0u, 0u, 0u, 0u);            // own entries 4q .. 4q+3
                if constexpr (4 * q < Q) m4 = *reinterpret_cast<const uint4*>(lists + w * Q + 4 * q);
                const uint32_t mine[4] = {m4.x, m4.y, m4.z, m4.w};
                static_for<0, 4>([&](auto e) {
                    constexpr int i = 4 * q + e;
                    x[i] = (w & 1) ? min(mine[e], theirs[e]) : max(mine[e], theirs[e]);
                });
            });
            bitonic_merge_desc<QP>(x);
            __syncthreads();
            uint32_t* merged = lists + (w >> 1) * 2 * Q + ((w & 1) ? QP : 0);
            if ((w & 1) == 0) {
#pragma unroll
                for (int q = 0; q < QP / 4; ++q)
                    *reinterpret_cast<uint4*>(merged + 4 * q) =
                        make_uint4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
            } else {
#pragma unroll
                for (int q = 0; q < (2 * Q - QP) / 4; ++q)
                    *reinterpret_cast<uint4*>(merged + 4 * q) =
                        make_uint4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
            }
            __syncthreads();
            T = kth_of_two_lists<2 * Q>(lists, lists + 2 * Q, k);
        } else {
            T = kth_of_two_lists<Q>(lists, lists + Q, k);
        }
    }

    // ---- kept sets: magnitude >= T, unless more than k magnitudes reach T (a tie at the
    // threshold): then only those above T, and the chunk goes through the whole-wavefront
    // pass that adds the lowest indices among the equals
    uint32_t own[NW];
    auto mark = [&](uint32_t thr) -> int {
#pragma unroll
        for (int j = 0; j < NW; ++j) own[j] = 0u;
        static_for<0, Q>([&](auto I) {
            constexpr int m = Q - 1 - I;   // descending so that shifting lands bit m at m
            own[m / 32] = push_if_at_least(own[m / 32], __float_as_uint(c[m]) & 0x7FFFFFFFu, thr);
        });
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            cnt += __popc(own[j]);
            s_mask[lane][w][j] = own[j];
        }
        s_cnt[lane][w] = static_cast<uint8_t>(cnt);
        __syncthreads();                          // also: every class is done with the lists
        int total = 0;
#pragma unroll
        for (int j = 0; j < W; ++j) total += s_cnt[lane][j];
        return total;
    };
    uint32_t thr_gt = T, thr_eq = 0xFFFFFFFFu;
    int need = 0;
    {
        const int cnt = mark(T);
        const bool tie = alive && cnt != k;      // the idle rows of a partial tile are all zero
        if (__syncthreads_or(tie ? 1 : 0)) {
            if (tie) {
                thr_gt = T + 1u;     // <= 0x80000000: no magnitude reaches that
                thr_eq = T;
            }
            const int above = mark(thr_gt);
            if (tie) need = k - above;
            // the tied chunks' coefficients in natural order in their rows, for wavefront 0
#pragma unroll
            for (int m = 0; m < Q; ++m) row[W * m + off] = c[m];
            __syncthreads();
            if (w == 0) {
                const unsigned long long tl = __ballot(need != 0);
                if (lane == 0) s_tie = tl;
                emit_tied_chunks<S / 32, kWave>(buf, p, lane, need, thr_gt, thr_eq, chunk0, idx_out,
                                                val_out, nullptr);
            }
            __syncthreads();
            if (need != 0) {
#pragma unroll
                for (int m = 0; m < Q; ++m) c[m] = row[W * m + off];   // alpha_j * remainder
            }
            __syncthreads();
        }
    }

    // ---- payload staging, remainder in (settled chunks).  The position of coefficient m of
    // this class is the number of kept coefficients of the chunk with a smaller index: the
    // class's own bits below m, and of another class w' its bits below m (+ 1 if that class's
    // offset is the smaller one).
    if (need == 0 && alive) {
        // the other classes' bits lined up with this class's steps, and counted into the start
        uint32_t plane0[NW], plane1[NW];
        uint32_t start = 0u;
#pragma unroll
        for (int j = 0; j < NW; ++j) plane0[j] = plane1[j] = 0u;
#pragma unroll
        for (int o = 1; o < W; ++o) {
            const int wo = (w + o) % W;
            const uint32_t adj = split_off<W>(wo) < off ? 1u : 0u;
            uint32_t ow[NW];
#pragma unroll
            for (int j = 0; j < NW; ++j) ow[j] = s_mask[lane][wo][j];
            start += ow[0] & adj;
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const uint32_t up = (j + 1 < NW) ? ow[j + 1] : 0u;
                const uint32_t sh = __builtin_amdgcn_alignbit(up, ow[j], adj);
                // add one-bit numbers into a two-bit counter per position
                const uint32_t carry = plane0[j] & sh;
                plane0[j] ^= sh;
                plane1[j] |= carry;
            }
        }
        char* lds = reinterpret_cast<char*>(buf);
        const uint32_t dump = static_cast<uint32_t>(sizeof(float)) *
                              (kRowDumps ? lane * kRow + G::kRowDump + (lane >> 4) : kTile + tid);
        uint32_t at = static_cast<uint32_t>(sizeof(float)) * (lane * kRow + start);
        const int idx0 = off;
        static_for<0, Q>([&](auto m) {
            const uint32_t kb = (own[m / 32] >> (m % 32)) & 1u;
            const uint32_t b0 = (plane0[m / 32] >> (m % 32)) & 1u;
            const bool keep = kb != 0u;
            const uint32_t a = keep ? at : dump;
            *reinterpret_cast<float*>(lds + a) = c[m];
            *reinterpret_cast<float*>(lds + a + sizeof(float) * kIdx0) =
                __int_as_float(idx0 + W * m);
            at += 4u * kb + 4u * b0;
            if constexpr (W == 4) at += 8u * ((plane1[m / 32] >> (m % 32)) & 1u);
            c[m] = (keep ? 0.0f : c[m]) * ((m == 0 && w == 0) ? p.alpha0 : p.alpha);
        });
    }
    __syncthreads();
    {
        // the tile's 64*k entries are contiguous in both payload arrays
        const uint32_t magic = entry_magic(k);
        const unsigned long long tie_chunks = s_tie;
        float* vo = val_out + chunk0 * k;
        int32_t* io = idx_out + chunk0 * k;
        if (k % 4 == 0) {
            const int quads = live * k / 4;                // 16-byte pieces of the tile
            for (int q = tid; q < quads; q += kThreads) {
                const uint32_t e = 4u * static_cast<uint32_t>(q);
                const uint32_t r = __umulhi(e, magic);     // chunk of the tile, k >= 4
                const uint32_t j = e - r * static_cast<uint32_t>(k);
                if ((tie_chunks >> r) & 1ull) continue;    // written by the tie pass
                const float* src = &buf[r * kRow + j];
                st_f4<false>(vo + e, *reinterpret_cast<const float4*>(src));
                const float4 iv = *reinterpret_cast<const float4*>(src + kIdx0);
                *reinterpret_cast<int4*>(io + e) =
                    make_int4(__float_as_int(iv.x), __float_as_int(iv.y), __float_as_int(iv.z),
                              __float_as_int(iv.w));
            }
        } else {
            // four entries of a lane could straddle two chunks (and the arrays need not be
            // 16-byte aligned): one entry per lane
            for (uint32_t e = tid; e < static_cast<uint32_t>(live * k); e += kThreads) {
                const uint32_t r = (k == 1) ? e : __umulhi(e, magic);
                const uint32_t j = e - r * static_cast<uint32_t>(k);
                if ((tie_chunks >> r) & 1ull) continue;
                const float* src = &buf[r * kRow + j];
                vo[e] = src[0];
                io[e] = __float_as_int(src[kIdx0]);
            }
        }
    }
    __syncthreads();

    // ---- new momentum = inverse transform of the remainder
    split_inverse_to_rows<S, W>(row, w, c);
    {
        constexpr int kIt = Q / 4;
        if (!partial) {
#pragma unroll 4
            for (int it = 0; it < kIt; ++it) {
                const int e4 = 4 * (tid + kThreads * it);
                const int r = e4 / S, col = e4 - r * S;
                st_f4<false>(mom + base + e4, split_output<S, W>(&buf[r * kRow], col));
            }
        } else {
            for (int it = 0; it < kIt; ++it) {
                const int e4 = 4 * (tid + kThreads * it);
                const int r = e4 / S, col = e4 - r * S;
                const int64_t i0 = base + e4;
                if (i0 + 3 < n) {
                    st_f4<false>(mom + i0, split_output<S, W>(&buf[r * kRow], col));
                } else if (i0 < n) {
                    const float4 y = split_output<S, W>(&buf[r * kRow], col);
                    const float v[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (i0 + j < n) mom[i0 + j] = v[j];
                }
            }
        }
    }
}

// Decompress-and-update half (transmitted indices, DCT domain, fp32 values + int32 indices) on
// full tiles of 64 chunks, W wavefronts per workgroup.
//
// Scatter-add: wavefront w owns the rows [64w/W, 64(w+1)/W) of the tile, so no two wavefronts
// ever add into the same accumulator and, inside a wavefront, LDS operations complete in program
// order: replica after replica, deterministic.  k a multiple of 4: 16-byte loads of four
// consecutive entries of one chunk per lane, a batch of four replicas requested at a time and
// the next batch before the current one is applied (two batches in flight per wavefront: the
// wavefronts of a workgroup are in this phase together, so what each keeps in flight decides
// how busy the memory is); a plain read-add-write when the four indices of every lane and the
// step from the previous lane ascend strictly (what compress emits), LDS atomics otherwise
// (duplicates add).
// Other k: one entry per lane, LDS atomics.  Then every class gathers its coefficients from
// the rows, the inverse transform runs as in compress_split, and all wavefronts stream the
// parameters (and the moments of Decoupled AdamW) through the update.
template <int S, int W, bool PARAM_BF16>
__global__ __launch_bounds__(kWave * W) void decompress_split(
    KParams p, int64_t tiles, int64_t n, int64_t n_chunks, const int32_t* __restrict__ idx,
    int64_t idx_stride, const float* __restrict__ val, int64_t val_stride,
    void* __restrict__ params, AdamPtrs ad, float* __restrict__ presign_dbg) {
    using G = SplitGeom<S, W>;
    constexpr int Q = G::Q, kRow = G::kRow, kThreads = G::kThreads, kTile = G::kTile;
    constexpr int kRowsPerWave = kWave / W;
    __shared__ __attribute__((aligned(16))) float buf[kTile];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k = p.k;

    // full tiles, then one partial tile of the chunks left over, the last of them possibly
    // ragged (as in compress_split)
    const int64_t tile = blockIdx.x;
    const bool partial = tile >= tiles;    // (a partial tile can have 64 rows, the last ragged)
    const int live = partial ? static_cast<int>(n_chunks - tiles * kWave) : kWave;
    // rows of this wavefront's share that are chunks
    const int my_rows = min(max(live - w * kRowsPerWave, 0), kRowsPerWave);
    const int64_t base = tile * static_cast<int64_t>(kWave * S);
    float* row = &buf[lane * kRow];

    // ---- the tile's bf16 parameters, requested first: they are needed only after the
    // transform (plain update of a full tile.  fp32 parameters, or the moments of Decoupled
    // AdamW, held that long would cost a wavefront per SIMD in registers: they are loaded
    // where they are used)
    constexpr int kPieces = Q / 4;                // 4-element pieces of the tile per thread
    uint2 early[kPieces];
    const bool params_early = PARAM_BF16 && !partial && !p.adam;
    if constexpr (PARAM_BF16) {
        if (params_early) {
#pragma unroll
            for (int it = 0; it < kPieces; ++it)
                early[it] = ld_u2<true>(static_cast<const uint16_t*>(params) + base +
                                        4 * (tid + kThreads * it));
        }
    }

    // ---- zero this wavefront's rows
    {
        float* mine = &buf[w * kRowsPerWave * kRow];
        for (int v = lane; v < kRowsPerWave * kRow / 4; v += kWave)
            *reinterpret_cast<float4*>(mine + 4 * v) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    wave_lds_sync();

    // ---- scatter-add of this wavefront's rows, replica after replica
    {
        const int64_t entry0 = (tile * kWave + w * kRowsPerWave) * static_cast<int64_t>(k);
        float* rows = &buf[w * kRowsPerWave * kRow];
        const uint32_t magic = entry_magic(k);
        if (k % 4 == 0) {
            const int quads = my_rows * k / 4;             // 16-byte pieces per replica
            constexpr int kBatch = 4;                      // replicas per batch
            // A step = one batch of replicas for one group of 64 pieces.  The loads of the
            // next step are requested before the current one is applied: two batches in
            // flight per wavefront.
            const int n_batches = (p.R + kBatch - 1) / kBatch;
            const int steps = ((quads + kWave - 1) / kWave) * n_batches;
            auto piece = [&](int t, uint32_t& e, bool& in) {
                const int q = (t / n_batches) * kWave + lane;
                in = q < quads;
                e = 4u * static_cast<uint32_t>(in ? q : 0);
            };
            auto request = [&](int t, int4 (&iv)[kBatch], float4 (&vv)[kBatch]) {
                uint32_t e;
                bool in;
                piece(t, e, in);
                const int r0 = (t % n_batches) * kBatch;
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    if (r0 + b < p.R && in) {
                        const uint4 x = ld_u4<true>(idx + (r0 + b) * idx_stride + entry0 + e);
                        iv[b] = make_int4(static_cast<int>(x.x), static_cast<int>(x.y),
                                          static_cast<int>(x.z), static_cast<int>(x.w));
                        vv[b] = ld_f4<true>(val + (r0 + b) * val_stride + entry0 + e);
                    } else {
                        iv[b] = make_int4(-1, -1, -1, -1);
                        vv[b] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    }
                }
            };
            auto apply = [&](int t, const int4 (&iv)[kBatch], const float4 (&vv)[kBatch]) {
                uint32_t e;
                bool in;
                piece(t, e, in);
                const int r0 = (t % n_batches) * kBatch;
                const uint32_t r = (k == 4) ? (e >> 2) : __umulhi(e, magic);   // row of the wavefront
                const bool chunk_start = (e - r * static_cast<uint32_t>(k)) == 0u;
                float* arow = rows + r * kRow;
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    if (r0 + b < p.R) {
                        const int at[4] = {iv[b].x, iv[b].y, iv[b].z, iv[b].w};
                        const float v[4] = {vv[b].x, vv[b].y, vv[b].z, vv[b].w};
                        const int prev = __shfl_up(at[3], 1);
                        const bool asc = at[0] < at[1] && at[1] < at[2] && at[2] < at[3] &&
                                         (lane == 0 || chunk_start || prev < at[0]);
                        if (__any(in && !asc)) {
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                if (static_cast<uint32_t>(at[c]) < static_cast<uint32_t>(S))
                                    atomicAdd(&arow[at[c]], v[c]);
                        } else {
                            float old[4];
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                old[c] = (static_cast<uint32_t>(at[c]) < static_cast<uint32_t>(S))
                                             ? arow[at[c]] : 0.0f;
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                if (static_cast<uint32_t>(at[c]) < static_cast<uint32_t>(S))
                                    arow[at[c]] = old[c] + v[c];
                        }
                        wave_lds_sync();
                    }
                }
            };
            int4 iv0[kBatch], iv1[kBatch];
            float4 vv0[kBatch], vv1[kBatch];
            if (steps > 0) request(0, iv0, vv0);
            for (int t = 0; t < steps; t += 2) {
                if (t + 1 < steps) request(t + 1, iv1, vv1);
                apply(t, iv0, vv0);
                if (t + 2 < steps) request(t + 2, iv0, vv0);
                if (t + 1 < steps) apply(t + 1, iv1, vv1);
            }
        } else {
            // one entry per lane, LDS atomics; four groups of 64 entries requested together
            const int entries = my_rows * k;
            constexpr int kGroups = 4;
            for (int r = 0; r < p.R; ++r) {
                const int32_t* ir = idx + r * idx_stride + entry0;
                const float* vr = val + r * val_stride + entry0;
                for (int e0 = 0; e0 < entries; e0 += kGroups * kWave) {
                    int at[kGroups];
                    float v[kGroups];
#pragma unroll
                    for (int g = 0; g < kGroups; ++g) {
                        const int e = e0 + g * kWave + lane;
                        at[g] = -1;
                        v[g] = 0.0f;
                        if (e < entries) {
                            at[g] = ir[e];
                            v[g] = vr[e];
                        }
                    }
#pragma unroll
                    for (int g = 0; g < kGroups; ++g) {
                        const int e = e0 + g * kWave + lane;
                        const uint32_t rr = (k == 1) ? static_cast<uint32_t>(e)
                                                     : __umulhi(static_cast<uint32_t>(e), magic);
                        if (e < entries && static_cast<uint32_t>(at[g]) < static_cast<uint32_t>(S))
                            atomicAdd(&rows[rr * kRow + at[g]], v[g]);
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- the lane's class of the averaged coefficients: a[W*m + off] * alpha_j / R
    const int off = split_off<W>(w);
    const float scale = p.alpha * p.inv_R;
    float c[Q];
    {
        const float* src = row + off;
#pragma unroll
        for (int m = 0; m < Q; ++m) c[m] = src[W * m] * scale;
        if (w == 0) c[0] = row[0] * (p.alpha0 * p.inv_R);
    }
    __syncthreads();
    split_inverse_to_rows<S, W>(row, w, c);

    // ---- y out of the rows, optional sign, parameter update, coalesced; the parameters (and
    // moments) of a batch of iterations are requested before the first is used
    {
        constexpr int kIt = Q / 4;                // 16-byte pieces per thread
        constexpr int kBatch = (kIt % 8 == 0) ? 8 : 4;
        static_assert(kIt % kBatch == 0, "whole batches");
        // (full tiles run the code without the checks against the end of the shard: with them
        // the loads of a batch are no longer issued together)
        auto update = [&](auto guarded_tag) {
        constexpr bool kGuarded = decltype(guarded_tag)::value;
#pragma unroll 1
        for (int b0 = 0; b0 < kIt; b0 += kBatch) {
            float4 old4[kBatch], m4[kBatch], v4[kBatch], x4[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int64_t i = base + 4 * (tid + kThreads * (b0 + j));
                if constexpr (kGuarded) {
                    old4[j] = m4[j] = v4[j] = x4[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    if (i + 3 >= n) continue;   // the shard's end: handled below
                }
                if constexpr (PARAM_BF16) {
                    const uint2 pb = ld_u2<true>(static_cast<const uint16_t*>(params) + i);
                    old4[j] = make_float4(__uint_as_float(pb.x << 16),
                                          __uint_as_float(pb.x & 0xFFFF0000u),
                                          __uint_as_float(pb.y << 16),
                                          __uint_as_float(pb.y & 0xFFFF0000u));
                } else {
                    old4[j] = ld_f4<true>(static_cast<const float*>(params) + i);
                }
                x4[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (p.adam) {
                    m4[j] = ld_f4<true>(ad.m + i);
                    v4[j] = ld_f4<true>(ad.v + i);
                    if (p.amsgrad) x4[j] = ld_f4<true>(ad.vmax + i);
                }
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int e4 = 4 * (tid + kThreads * (b0 + j));
                const int r = e4 / S, col = e4 - r * S;
                const int64_t i = base + e4;
                if (kGuarded && i + 3 >= n) {
                    // the piece that straddles the end of the shard: element by element
                    if (i < n) {
                        const float4 y4 = split_output<S, W>(&buf[r * kRow], col);
                        const float yv[4] = {y4.x, y4.y, y4.z, y4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if (i + e >= n) break;
                            if (presign_dbg) presign_dbg[i + e] = yv[e];
                            const float q = sign_or_self(yv[e], p.use_sign);
                            const float th = PARAM_BF16
                                ? bf16_to_f32(static_cast<const uint16_t*>(params)[i + e])
                                : static_cast<const float*>(params)[i + e];
                            float nw;
                            if (p.adam) {
                                float vm = p.amsgrad ? ad.vmax[i + e] : 0.0f;
                                nw = adamw_step(p, th, q, ad.m[i + e], ad.v[i + e], vm);
                                if (p.amsgrad) ad.vmax[i + e] = vm;
                            } else {
                                nw = fmaf(-p.lr, q, th * p.wd_scale);
                            }
                            if constexpr (PARAM_BF16)
                                static_cast<uint16_t*>(params)[i + e] = f32_to_bf16(nw);
                            else
                                static_cast<float*>(params)[i + e] = nw;
                        }
                    }
                    continue;
                }
                const float4 y4 = split_output<S, W>(&buf[r * kRow], col);
                if (presign_dbg) st_f4<false>(presign_dbg + i, y4);
                const float y[4] = {y4.x, y4.y, y4.z, y4.w};
                const float old[4] = {old4[j].x, old4[j].y, old4[j].z, old4[j].w};
                float nw[4];
                if (p.adam) {
                    float m[4] = {m4[j].x, m4[j].y, m4[j].z, m4[j].w};
                    float v[4] = {v4[j].x, v4[j].y, v4[j].z, v4[j].w};
                    float x[4] = {x4[j].x, x4[j].y, x4[j].z, x4[j].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        nw[e] = adamw_step(p, old[e], sign_or_self(y[e], p.use_sign), m[e], v[e], x[e]);
                    st_f4<true>(ad.m + i, make_float4(m[0], m[1], m[2], m[3]));
                    st_f4<true>(ad.v + i, make_float4(v[0], v[1], v[2], v[3]));
                    if (p.amsgrad) st_f4<true>(ad.vmax + i, make_float4(x[0], x[1], x[2], x[3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        nw[e] = fmaf(-p.lr, sign_or_self(y[e], p.use_sign), old[e] * p.wd_scale);
                }
                if constexpr (PARAM_BF16) {
                    uint2 o;
                    o.x = pack_bf16x2(nw[0], nw[1]);
                    o.y = pack_bf16x2(nw[2], nw[3]);
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(params) + i) = o;
                } else {
                    st_f4<true>(static_cast<float*>(params) + i,
                                make_float4(nw[0], nw[1], nw[2], nw[3]));
                }
            }
        }
        };
        if (params_early) {
#pragma unroll
            for (int it = 0; it < kPieces; ++it) {
                const int e4 = 4 * (tid + kThreads * it);
                const int r = e4 / S, col = e4 - r * S;
                const int64_t i = base + e4;
                const float4 y4 = split_output<S, W>(&buf[r * kRow], col);
                if (presign_dbg) st_f4<false>(presign_dbg + i, y4);
                const float y[4] = {y4.x, y4.y, y4.z, y4.w};
                const float old[4] = {__uint_as_float(early[it].x << 16),
                                      __uint_as_float(early[it].x & 0xFFFF0000u),
                                      __uint_as_float(early[it].y << 16),
                                      __uint_as_float(early[it].y & 0xFFFF0000u)};
                float nw[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    nw[e] = fmaf(-p.lr, sign_or_self(y[e], p.use_sign), old[e] * p.wd_scale);
                uint2 o;
                o.x = pack_bf16x2(nw[0], nw[1]);
                o.y = pack_bf16x2(nw[2], nw[3]);
                *reinterpret_cast<uint2*>(static_cast<uint16_t*>(params) + i) = o;
            }
        } else if (partial) {
            update(std::true_type{});
        } else {
            update(std::false_type{});
        }
    }
}

}  // namespace deto
