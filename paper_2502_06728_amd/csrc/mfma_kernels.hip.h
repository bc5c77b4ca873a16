// Matrix-core kernels for the (chunk size, k) pairs the lane-per-chunk and two-lanes-per-chunk
// kernels do not cover (chunk sizes 32 ... 224 in steps of 32, any k, top-k selection): the DCT
// of Algorithm 1 as the dense product it is defined as, on v_mfma_f32_32x32x2f32.
//
// One wavefront (= one workgroup) owns a tile of 32 complete chunks, held as a 32 x S matrix
// in LDS (row = chunk).  With X the tile and D the S x S DCT-II matrix:
//     coefficients^T = D   * X^T      (A operand: D rows,     B operand: X rows)
//     output^T       = D^T * A_in^T   (A operand: D columns,  B operand: coefficient rows)
// so both directions read their B operand from the LDS rows with the same 16-byte reads
// (contraction index 8q + 4h + i for half-wave h at MFMA step 4q + i) and differ only in how
// the A operand walks the cosine table  tab[t] = cos(pi t / (2S)), t in [0, 4S):
//     D[j][n] = alpha_j * tab[(2n+1) j mod 4S].
// The scale alpha_j is applied outside the product.  Selection is a bitwise binary search
// for the k-th largest magnitude of each chunk (two lanes per chunk, half a row each),
// followed by one pass over the chunks with the whole wavefront that emits the payload in
// ascending index order and leaves alpha_j * (what the receivers will not get) in LDS for
// the inverse product: the new momentum is the inverse transform of that remainder.
#pragma once

#include "deto_device.hip.h"
#include "generic_kernels.hip.h"

namespace deto {

typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kMfmaChunks = 32;   // chunks per tile = N of the 32x32 MFMA

template <int NB>
struct MfmaGeom {
    static constexpr int S = 32 * NB;          // chunk size
    static constexpr int kRow = S + 4;         // floats per LDS row (16 B of padding)
    static constexpr int kTab = 4 * S;         // cosine table entries
    static constexpr int kVecIters = S / 8;    // 16-byte pieces per lane in a linear pass
    static constexpr size_t kSmemBytes = sizeof(float) * (kMfmaChunks * kRow + kTab);
    // wavefronts per SIMD the LDS leaves room for (160 KB per CU, 4 SIMDs): the register
    // allocation is held to that occupancy
    static constexpr int kWavesPerSimd = (NB <= 6) ? 2 : 1;
};

// tab[t] = cos(pi t / (2S)) for t in [0, 4S), from the first quarter period by symmetry
template <int S>
__device__ __forceinline__ void build_cos_table_quarter(float* tab, int lane) {
    for (int t = lane; t <= S; t += kWave) {
        float c = static_cast<float>(cos(3.14159265358979323846 * static_cast<double>(t) /
                                         (2.0 * static_cast<double>(S))));
        if (t == S) c = 0.0f;
        tab[t] = c;
        tab[2 * S - t] = -c;
        tab[2 * S + t] = -c;
        if (t > 0) tab[4 * S - t] = c;
    }
}

__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// Which coefficient / element indices a lane holds after a product.  Lane (t, h) of the
// wavefront owns, of chunk t, the groups of GS consecutive indices 2*GS*G + GS*h + e
// (G = 0 .. kGroups-1, e < GS): its partner lane t + 32*(1-h) owns the other half.
// Chunk sizes that are a multiple of 64 use the symmetry of the cosine (below), which pairs
// each even index with the odd one after it: GS = 8.
template <int NB>
struct MfmaOwn {
    static constexpr bool kHalf = (NB % 2 == 0);
    static constexpr int GS = kHalf ? 8 : 4;
    static constexpr int kGroups = 16 * NB / GS;
};

__device__ __forceinline__ void zero_acc(f32x16_t& a) {
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = 0.0f;
}

// One contraction step for all NB output blocks: blocks below HB take b_lo, the others b_hi.
template <int NB, int HB>
__device__ __forceinline__ void mfma_step(const float* __restrict__ tab, int (&cur)[NB],
                                          const int (&inc)[NB], const int (&inc5)[NB],
                                          f32x16_t (&acc)[NB], float b_lo, float b_hi, bool last) {
    constexpr int W = 4 * 32 * NB;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const float a = tab[cur[b]];
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b < HB ? b_lo : b_hi, acc[b], 0, 0, 0);
        const int nx = cur[b] + (last ? inc5[b] : inc[b]);
        cur[b] = nx >= W ? nx - W : nx;
    }
}

// Forward transform of the tile: row t of `buf` (chunk t, m1) is replaced by its DCT-II
// coefficients c; mag[] receives the magnitudes (bit patterns) of the coefficients this lane
// owns, in ascending index order.
//
// NB odd:  coefficients^T = D * X^T with all S contraction steps.
// NB even: cos(pi (2(S-1-n)+1) j / (2S)) = (-1)^j cos(pi (2n+1) j / (2S)), so even rows only
//          see u_n = x_n + x_{S-1-n} and odd rows w_n = x_n - x_{S-1-n}, n < S/2: half the
//          contraction length.  Blocks [0, NB/2) hold rows 2m, blocks [NB/2, NB) rows 2m+1.
template <int NB>
__device__ __forceinline__ void forward_to_lds(float* __restrict__ buf,
                                               const float* __restrict__ tab, const KParams& p,
                                               int t, int h, uint32_t (&mag)[NB * 16]) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow, W = G::kTab;
    f32x16_t acc[NB];
    int cur[NB], inc[NB], inc5[NB];
    float* row = &buf[t * kRow];
    if constexpr (!MfmaOwn<NB>::kHalf) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int j = 32 * b + t;
            cur[b] = ((8 * h + 1) * j) % W;     // contraction index n = 4h first
            inc[b] = 2 * j;
            inc5[b] = (10 * j) % W;
            zero_acc(acc[b]);
        }
#pragma unroll 1
        for (int q = 0; q < S / 8; ++q) {
            const float4 x = *reinterpret_cast<const float4*>(row + 8 * q + 4 * h);
            const float xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mfma_step<NB, NB>(tab, cur, inc, inc5, acc, xv[i], xv[i], i == 3);
        }
        wave_lds_sync();
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int j0 = 32 * b + 8 * g4 + 4 * h;
                float c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    c[i] = acc[b][4 * g4 + i] * p.alpha;
                    if (b == 0 && g4 == 0 && i == 0 && h == 0) c[i] = acc[0][0] * p.alpha0;
                    mag[16 * b + 4 * g4 + i] = __float_as_uint(c[i]) & 0x7FFFFFFFu;
                }
                *reinterpret_cast<float4*>(row + j0) = make_float4(c[0], c[1], c[2], c[3]);
            }
        }
    } else {
        constexpr int HB = NB / 2;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int j = (b < HB) ? 2 * (32 * b + t) : 2 * (32 * (b - HB) + t) + 1;
            cur[b] = ((8 * h + 1) * j) % W;
            inc[b] = 2 * j;
            inc5[b] = (10 * j) % W;
            zero_acc(acc[b]);
        }
#pragma unroll 1
        for (int q = 0; q < S / 16; ++q) {
            const float4 xa = *reinterpret_cast<const float4*>(row + 8 * q + 4 * h);
            const float4 xb = *reinterpret_cast<const float4*>(row + S - 8 * q - 4 * h - 4);
            const float u[4] = {xa.x + xb.w, xa.y + xb.z, xa.z + xb.y, xa.w + xb.x};
            const float w[4] = {xa.x - xb.w, xa.y - xb.z, xa.z - xb.y, xa.w - xb.x};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mfma_step<NB, HB>(tab, cur, inc, inc5, acc, u[i], w[i], i == 3);
        }
        wave_lds_sync();
        // acc[b][r], b < HB, is coefficient 2m and acc[b + HB][r] coefficient 2m + 1 with
        // m = 32b + 8(r/4) + 4h + r%4: eight consecutive coefficients per (b, r/4)
#pragma unroll
        for (int b = 0; b < HB; ++b) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int j0 = 64 * b + 16 * g4 + 8 * h;
                const int Gp = 4 * b + g4;
                float c[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    c[2 * i] = acc[b][4 * g4 + i] * p.alpha;
                    c[2 * i + 1] = acc[b + HB][4 * g4 + i] * p.alpha;
                }
                if (b == 0 && g4 == 0 && h == 0) c[0] = acc[0][0] * p.alpha0;
#pragma unroll
                for (int e = 0; e < 8; ++e) mag[8 * Gp + e] = __float_as_uint(c[e]) & 0x7FFFFFFFu;
                *reinterpret_cast<float4*>(row + j0) = make_float4(c[0], c[1], c[2], c[3]);
                *reinterpret_cast<float4*>(row + j0 + 4) = make_float4(c[4], c[5], c[6], c[7]);
            }
        }
    }
}

// Inverse transform of the tile: row t of `buf` holds a_j' = alpha_j a_j (the scale already
// applied, or applied by `post`); it is replaced by post(sum_j a_j' cos(pi (2n+1) j / (2S))).
//
// NB even: with E_n the sum over even j and O_n the sum over odd j, y_n = E_n + O_n and
//          y_{S-1-n} = E_n - O_n, so only n < S/2 is computed, each half with S/2 steps.
//          Blocks [0, NB/2) accumulate E for n = 32b + t, blocks [NB/2, NB) accumulate O.
template <int NB, class Post>
__device__ __forceinline__ void inverse_to_lds(float* __restrict__ buf,
                                               const float* __restrict__ tab, int t, int h,
                                               Post post) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow, W = G::kTab;
    f32x16_t acc[NB];
    int cur[NB], inc[NB], inc5[NB];
    float* row = &buf[t * kRow];
    if constexpr (!MfmaOwn<NB>::kHalf) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int m2 = 2 * (32 * b + t) + 1;
            cur[b] = (m2 * 4 * h) % W;          // contraction index j = 4h first
            inc[b] = m2;
            inc5[b] = (5 * m2) % W;
            zero_acc(acc[b]);
        }
#pragma unroll 1
        for (int q = 0; q < S / 8; ++q) {
            const float4 x = *reinterpret_cast<const float4*>(row + 8 * q + 4 * h);
            const float xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mfma_step<NB, NB>(tab, cur, inc, inc5, acc, xv[i], xv[i], i == 3);
        }
        wave_lds_sync();
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int n0 = 32 * b + 8 * g4 + 4 * h;
                *reinterpret_cast<float4*>(row + n0) =
                    make_float4(post(acc[b][4 * g4]), post(acc[b][4 * g4 + 1]),
                                post(acc[b][4 * g4 + 2]), post(acc[b][4 * g4 + 3]));
            }
        }
    } else {
        constexpr int HB = NB / 2;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int m2 = 2 * (32 * (b < HB ? b : b - HB) + t) + 1;
            cur[b] = (((b < HB) ? 8 * h : 8 * h + 1) * m2) % W;   // j = 2*4h (+1) first
            inc[b] = 2 * m2;
            inc5[b] = (10 * m2) % W;
            zero_acc(acc[b]);
        }
#pragma unroll 1
        for (int q = 0; q < S / 16; ++q) {
            const float4 lo = *reinterpret_cast<const float4*>(row + 16 * q + 8 * h);
            const float4 hi = *reinterpret_cast<const float4*>(row + 16 * q + 8 * h + 4);
            const float ev[4] = {lo.x, lo.z, hi.x, hi.z};
            const float od[4] = {lo.y, lo.w, hi.y, hi.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mfma_step<NB, HB>(tab, cur, inc, inc5, acc, ev[i], od[i], i == 3);
        }
        wave_lds_sync();
#pragma unroll
        for (int b = 0; b < HB; ++b) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int n0 = 32 * b + 8 * g4 + 4 * h;
                float lo4[4], hi4[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float e = acc[b][4 * g4 + i], o = acc[b + HB][4 * g4 + i];
                    lo4[i] = post(e + o);       // element n0 + i
                    hi4[i] = post(e - o);       // element S - 1 - (n0 + i)
                }
                *reinterpret_cast<float4*>(row + n0) = make_float4(lo4[0], lo4[1], lo4[2], lo4[3]);
                *reinterpret_cast<float4*>(row + S - 4 - n0) =
                    make_float4(hi4[3], hi4[2], hi4[1], hi4[0]);
            }
        }
    }
}

// ---- tile streaming and bookkeeping shared by the 32-chunk-tile kernels (NB = S / 32)

// m1 = beta*m + g for the tile's 32*S contiguous elements, coalesced, into the LDS rows (deep
// unroll: nothing else of this wavefront is in flight, so the loads of half a tile or more are
// issued at once)
template <int NB, bool GRAD_BF16>
__device__ __forceinline__ void fold_tile_rows(float* __restrict__ buf, const KParams& p, int lane,
                                               const void* __restrict__ grad,
                                               const float* __restrict__ mom, int64_t base) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow;
#pragma unroll 16
    for (int it = 0; it < G::kVecIters; ++it) {
        const int e4 = 4 * (lane + kWave * it);
        const int row = e4 / S, col = e4 - row * S;
        const float4 m = ld_f4<false>(mom + base + e4);
        float4 g;
        if constexpr (GRAD_BF16) {
            const uint2 gb = ld_u2<false>(static_cast<const uint16_t*>(grad) + base + e4);
            g = make_float4(__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xFFFF0000u),
                            __uint_as_float(gb.y << 16), __uint_as_float(gb.y & 0xFFFF0000u));
        } else {
            g = ld_f4<false>(static_cast<const float*>(grad) + base + e4);
        }
        const float4 x = make_float4(fmaf(p.beta, m.x, g.x), fmaf(p.beta, m.y, g.y),
                                     fmaf(p.beta, m.z, g.z), fmaf(p.beta, m.w, g.w));
        *reinterpret_cast<float4*>(&buf[row * kRow + col]) = x;
    }
}

// the LDS rows (new momentum) out, coalesced
template <int NB>
__device__ __forceinline__ void store_tile_rows(const float* __restrict__ buf, int lane,
                                                float* __restrict__ mom, int64_t base) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow;
#pragma unroll 4
    for (int it = 0; it < G::kVecIters; ++it) {
        const int e4 = 4 * (lane + kWave * it);
        const int row = e4 / S, col = e4 - row * S;
        st_f4<false>(mom + base + e4, *reinterpret_cast<const float4*>(&buf[row * kRow + col]));
    }
}

// Chunks with ties at the k-th magnitude (need != 0 on the chunk's lanes), one at a time with
// the whole wavefront; their LDS rows hold the coefficients (ROWS rows; lane tt of the calling
// wavefront carries chunk tt's need and thresholds).  Everything above thr_eq is kept
// and, of the entries equal to it, the `need` lowest indices.  The payload goes out and the
// row is left holding alpha_j * remainder.
template <int NB, int ROWS = kMfmaChunks>
__device__ __forceinline__ void emit_tied_chunks(float* __restrict__ buf, const KParams& p,
                                                 int lane, int need, uint32_t thr_gt,
                                                 uint32_t thr_eq, int64_t chunk0,
                                                 void* __restrict__ idx_out,
                                                 void* __restrict__ val_out,
                                                 float* __restrict__ coeff_dbg) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow;
    const int k = p.k;
    if (!__any(need != 0)) return;
    for (int tt = 0; tt < ROWS; ++tt) {
        const int c_need = __builtin_amdgcn_readlane(need, tt);
        if (c_need == 0) continue;
        const uint32_t c_gt = __builtin_amdgcn_readlane(thr_gt, tt);
        const uint32_t c_eq = __builtin_amdgcn_readlane(thr_eq, tt);
        const int64_t chunk = chunk0 + tt;
        int kept_before = 0, eq_before = 0;
#pragma unroll
        for (int e0 = 0; e0 < S; e0 += kWave) {
            const int e = e0 + lane;
            const bool in = (S % kWave == 0) || e < S;
            const float c = in ? buf[tt * kRow + e] : 0.0f;
            const uint32_t mg = __float_as_uint(c) & 0x7FFFFFFFu;
            const bool eq = in && mg == c_eq;
            const uint64_t eqm = __ballot(eq);
            const int eq_rank = eq_before + lanes_below(eqm, lane);
            const bool keep = in && (mg >= c_gt || (eq && eq_rank < c_need));
            const uint64_t km = __ballot(keep);
            const int pos = kept_before + lanes_below(km, lane);
            float rem = c;
            if (keep && pos < k) {
                store_payload_index(idx_out, chunk * k + pos, p.idx_u8, e);
                store_payload_value(val_out, chunk * k + pos, p.val_dtype, c);
                rem = c - payload_roundtrip(p.val_dtype, c);
            }
            if (in) {
                if (coeff_dbg) coeff_dbg[chunk * S + e] = c;
                buf[tt * kRow + e] = rem * (e == 0 ? p.alpha0 : p.alpha);
            }
            kept_before += __popcll(km);
            eq_before += __popcll(eqm);
        }
    }
}

// Compress half on full tiles of 32 chunks (top-k selection, DCT domain).
template <int NB, bool GRAD_BF16>
__global__ __launch_bounds__(kWave)
__attribute__((amdgpu_waves_per_eu(MfmaGeom<NB>::kWavesPerSimd))) void compress_mfma(KParams p, int64_t tiles,
                                                       const void* __restrict__ grad,
                                                       float* __restrict__ mom,
                                                       void* __restrict__ idx_out,
                                                       void* __restrict__ val_out,
                                                       float* __restrict__ coeff_dbg) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow, W = G::kTab;
    __shared__ __attribute__((aligned(16))) float buf[kMfmaChunks * kRow];
    __shared__ float tab[W];

    const int lane = threadIdx.x;
    const int t = lane & 31, h = lane >> 5;
    const int k = p.k;
    build_cos_table_quarter<S>(tab, lane);
    wave_lds_sync();

    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t base = tile * static_cast<int64_t>(kMfmaChunks * S);
        const int64_t chunk0 = tile * kMfmaChunks;

        fold_tile_rows<NB, GRAD_BF16>(buf, p, lane, grad, mom, base);
        wave_lds_sync();

        // ---- DCT-II of every chunk of the tile, coefficients into the LDS rows
        uint32_t mag[NB * 16];
        forward_to_lds<NB>(buf, tab, p, t, h, mag);

        // ---- k-th largest magnitude of chunk t by binary search on its bits, counting in
        // registers: mag - cand is exact in 32 bits and its sign bit says "below cand"; the
        // sign bits are shifted into a collector word and counted 32 at a time.
        // thr_gt: everything at or above it is kept; thr_eq: of the entries equal to it the
        // first `need` (lowest indices) are kept as well.
        auto count_at_least = [&](uint32_t cand) -> int {
            int below = 0;
#pragma unroll
            for (int w = 0; w < NB * 16; w += 32) {
                uint32_t coll = 0u;
#pragma unroll
                for (int i = 0; i < 32 && w + i < NB * 16; ++i)
                    coll = __builtin_amdgcn_alignbit(coll, mag[w + i] - cand, 31);
                below += __popc(coll);
            }
            const int own = NB * 16 - below;
            return own + __shfl_xor(own, 32);
        };
        uint32_t T = 0u, thr_gt = 0u;
        bool done = false;
        for (int bit = 30; bit >= 0; --bit) {
            const uint32_t cand = T | (1u << bit);
            const int cnt = count_at_least(cand);
            if (!done && cnt >= k) {
                T = cand;
                if (cnt == k) {   // exactly k entries at or above cand: the selection is settled
                    done = true;
                    thr_gt = cand;
                }
            }
            if (__all(done)) break;
        }
        uint32_t thr_eq = 0xFFFFFFFFu;
        int need = 0;
        if (!__all(done)) {
            // lanes still open: T is the k-th largest magnitude itself
            const uint32_t gt = T + 1u;                       // <= 0x80000000: nothing reaches it
            const int cg_all = count_at_least(gt & 0x7FFFFFFFu);   // every lane takes part
            if (!done) {
                thr_gt = gt;
                thr_eq = T;
                need = k - ((gt > 0x7FFFFFFFu) ? 0 : cg_all);
            }
        }
        wave_lds_sync();

        // ---- payload out, remainder in.  Chunks whose search ended on an exact count
        // (need == 0: the kept set is "magnitude >= thr_gt") are finished by their two lanes
        // in parallel.  Lane (t, h) walks its index groups in ascending order, so the payload
        // position of an element is its rank among the lane's kept elements plus the partner
        // lane's kept elements with a smaller index: the partner's whole groups below G and,
        // for h = 1, its group G as well.  The partner's kept set comes over as a bit mask
        // (bit GS*G + e).
        {
            constexpr int GS = MfmaOwn<NB>::GS;
            constexpr int NW = (NB * 16 + 31) / 32;
            constexpr int kGroupsPerWord = 32 / GS;
            uint32_t other[NW];
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                uint32_t own = 0u;
#pragma unroll
                for (int r = 0; r < 32 && 32 * w + r < NB * 16; ++r)
                    own |= (mag[32 * w + r] >= thr_gt ? 1u : 0u) << r;
                other[w] = static_cast<uint32_t>(__shfl_xor(static_cast<int>(own), 32));
            }
            const bool settled = (need == 0);
            const int64_t cbase = (chunk0 + t) * k;
            float* row = &buf[t * kRow + GS * h];
            float* dbg = coeff_dbg ? coeff_dbg + (chunk0 + t) * S + GS * h : nullptr;
            int pos = 0;                       // kept so far: own and partner's lower groups
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const int left = MfmaOwn<NB>::kGroups - w * kGroupsPerWord;
                const int groups = left < kGroupsPerWord ? left : kGroupsPerWord;
                uint32_t ow = other[w];
#pragma unroll 2
                for (int gw = 0; gw < groups; ++gw) {
                    const int G = w * kGroupsPerWord + gw;
                    const int pk = __popc(ow & ((1u << GS) - 1u));   // partner's kept in group G
                    ow >>= GS;
                    if (h) pos += pk;
                    float c[GS], rem[GS];
#pragma unroll
                    for (int v = 0; v < GS / 4; ++v) {
                        const float4 c4 =
                            *reinterpret_cast<const float4*>(row + 2 * GS * G + 4 * v);
                        c[4 * v] = c4.x; c[4 * v + 1] = c4.y; c[4 * v + 2] = c4.z; c[4 * v + 3] = c4.w;
                    }
#pragma unroll
                    for (int e = 0; e < GS; ++e) {
                        const bool keep = (__float_as_uint(c[e]) & 0x7FFFFFFFu) >= thr_gt;
                        rem[e] = c[e];
                        if (settled && keep && pos < k) {
                            store_payload_index(idx_out, cbase + pos, p.idx_u8,
                                                2 * GS * G + GS * h + e);
                            store_payload_value(val_out, cbase + pos, p.val_dtype, c[e]);
                            rem[e] = c[e] - payload_roundtrip(p.val_dtype, c[e]);
                        }
                        pos += keep ? 1 : 0;
                        rem[e] *= (e == 0 && G == 0 && h == 0) ? p.alpha0 : p.alpha;
                    }
                    if (!h) pos += pk;
                    if (settled) {
#pragma unroll
                        for (int v = 0; v < GS / 4; ++v) {
                            if (dbg)
                                *reinterpret_cast<float4*>(dbg + 2 * GS * G + 4 * v) = make_float4(
                                    c[4 * v], c[4 * v + 1], c[4 * v + 2], c[4 * v + 3]);
                            *reinterpret_cast<float4*>(row + 2 * GS * G + 4 * v) = make_float4(
                                rem[4 * v], rem[4 * v + 1], rem[4 * v + 2], rem[4 * v + 3]);
                        }
                    }
                }
            }
        }
        wave_lds_sync();
        emit_tied_chunks<NB>(buf, p, lane, need, thr_gt, thr_eq, chunk0, idx_out, val_out, coeff_dbg);
        wave_lds_sync();

        // ---- new momentum = inverse transform of the remainder
        inverse_to_lds<NB>(buf, tab, t, h, [](float y) { return y; });
        wave_lds_sync();
        store_tile_rows<NB>(buf, lane, mom, base);
        wave_lds_sync();
    }
}

// Scatter-add of the tile's payload for fp32 values + int32 indices with k a multiple of 4:
// 16-byte loads (four consecutive entries of one chunk per lane), four of them in flight
// per lane and the next group of four requested before the current one is applied.  A
// group's read-add-write is batched (all reads, then all writes), which is exact when the
// entries of each chunk inside the group hit distinct addresses: checked as "indices ascend
// strictly from entry to entry within a chunk"; a group that fails the check is applied
// with LDS atomics instead.
template <int NB>
__device__ __forceinline__ void scatter_add_vec(float* __restrict__ buf, const KParams& p,
                                                int lane, const int32_t* __restrict__ idx,
                                                int64_t idx_stride,
                                                const float* __restrict__ val,
                                                int64_t val_stride, int64_t entry0,
                                                uint32_t magic) {
    constexpr int S = MfmaGeom<NB>::S, kRow = MfmaGeom<NB>::kRow;
    constexpr int GI = 4;                                  // 16-byte loads per lane and group
    const int k = p.k;
    const int quads = 8 * k;                               // 16-byte pieces per replica tile
    const int groups_per_rep = (quads + GI * kWave - 1) / (GI * kWave);
    const int total = p.R * groups_per_rep;

    int4 ia[GI], ib[GI];
    float4 va[GI], vb[GI];
    auto load = [&](int gi, int4 (&I)[GI], float4 (&V)[GI]) {
        const int r = gi / groups_per_rep, g = gi - r * groups_per_rep;
        const int32_t* ip = idx + r * idx_stride + entry0;
        const float* vp = val + r * val_stride + entry0;
#pragma unroll
        for (int i = 0; i < GI; ++i) {
            const int q = (g * GI + i) * kWave + lane;
            if (q < quads) {
                const uint4 t = ld_u4<true>(ip + 4 * q);
                I[i] = make_int4(static_cast<int>(t.x), static_cast<int>(t.y),
                                 static_cast<int>(t.z), static_cast<int>(t.w));
                V[i] = ld_f4<true>(vp + 4 * q);
            } else {
                I[i] = make_int4(-1, -1, -1, -1);
                V[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
    };

    load(0, ia, va);
    for (int gi = 0; gi < total; ++gi) {
        if (gi + 1 < total) load(gi + 1, ib, vb);
        const int g = gi % groups_per_rep;
        // iterations of this group that hold entries at all (wave-uniform)
        const int live = min(GI, (quads - g * GI * kWave + kWave - 1) / kWave);
        int rowbase[GI];
        bool bad = false;
#pragma unroll
        for (int i = 0; i < GI; ++i) {
            if (i >= live) break;
            const int q = (g * GI + i) * kWave + lane;
            const bool in = q < quads;
            const uint32_t e0 = 4u * static_cast<uint32_t>(q);
            const uint32_t row = __umulhi(e0, magic);
            const bool chunk_start = (e0 - row * static_cast<uint32_t>(k)) == 0u;
            rowbase[i] = static_cast<int>(row) * kRow;
            int prev = __shfl_up(ia[i].w, 1);
            if (i > 0) {
                const int wrap = __builtin_amdgcn_readlane(ia[i - 1].w, kWave - 1);
                if (lane == 0) prev = wrap;
            }
            const bool first = (i == 0 && lane == 0);      // nothing of this group before it
            const bool asc = ia[i].x < ia[i].y && ia[i].y < ia[i].z && ia[i].z < ia[i].w &&
                             (first || chunk_start || prev < ia[i].x);
            bad = bad || (in && !asc);
        }
        if (__any(bad)) {
#pragma unroll
            for (int i = 0; i < GI; ++i) {
                if (i >= live) break;
                const int at[4] = {ia[i].x, ia[i].y, ia[i].z, ia[i].w};
                const float v[4] = {va[i].x, va[i].y, va[i].z, va[i].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (static_cast<uint32_t>(at[c]) < static_cast<uint32_t>(S))
                        atomicAdd(&buf[rowbase[i] + at[c]], v[c]);
            }
        } else {
            float a[GI][4];
#pragma unroll
            for (int i = 0; i < GI; ++i) {
                if (i >= live) break;
                const int at[4] = {ia[i].x, ia[i].y, ia[i].z, ia[i].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    a[i][c] = (static_cast<uint32_t>(at[c]) < static_cast<uint32_t>(S))
                                  ? buf[rowbase[i] + at[c]] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < GI; ++i) {
                if (i >= live) break;
                const int at[4] = {ia[i].x, ia[i].y, ia[i].z, ia[i].w};
                const float v[4] = {va[i].x, va[i].y, va[i].z, va[i].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (static_cast<uint32_t>(at[c]) < static_cast<uint32_t>(S))
                        buf[rowbase[i] + at[c]] = a[i][c] + v[c];
            }
        }
        // the next group follows in program order: the LDS queue keeps the two apart
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < GI; ++i) {
            ia[i] = ib[i];
            va[i] = vb[i];
        }
    }
}

// Entry -> chunk inside a group of 8 chunks of k entries: floor(e / k) = umulhi(e, magic) with
// magic = ceil(2^32 / k), exact for e < 2^13 (k = 1 is the identity)
__device__ __forceinline__ uint32_t entry_magic(int k) {
    return (k == 1) ? 0u
                    : static_cast<uint32_t>(((1ull << 32) + static_cast<uint64_t>(k) - 1ull) /
                                            static_cast<uint64_t>(k));
}

// Zero the accumulator rows and scatter-add the tile's entries of all R replicas, replica
// after replica.  vec_scatter: fp32 values + int32 indices with k a multiple of 4 (16-byte
// loads); otherwise any payload format with 4-byte (or narrower) coalesced loads: the tile's
// entries of one replica are contiguous, four groups of 8 chunks run side by side (different
// LDS rows).  Within one instruction the entries of a chunk must hit distinct addresses for
// the plain read-add-write: guaranteed when their indices ascend strictly, else LDS atomics.
template <int NB>
__device__ __forceinline__ void scatter_tile(float* __restrict__ buf, const KParams& p, int lane,
                                             int vec_scatter, const void* __restrict__ idx,
                                             int64_t idx_stride, const void* __restrict__ val,
                                             int64_t val_stride, int64_t entry0, uint32_t magic) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow;
    const int k = p.k;
    const uint32_t group_entries = 8u * static_cast<uint32_t>(k);
    const int scatter_iters = static_cast<int>((group_entries + kWave - 1) / kWave);
    for (int v = lane; v < kMfmaChunks * kRow / 4; v += kWave)
        *reinterpret_cast<float4*>(&buf[4 * v]) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    wave_lds_sync();

    // ---- scatter-add, replica after replica.  The tile's entries of one replica are
    // contiguous; four groups of 8 chunks run side by side (different LDS rows).  Within
    // one instruction the entries of a chunk must hit distinct addresses for the plain
    // read-add-write: guaranteed when their indices ascend strictly, else LDS atomics.
    if (vec_scatter)
        scatter_add_vec<NB>(buf, p, lane, static_cast<const int32_t*>(idx), idx_stride,
                            static_cast<const float*>(val), val_stride, entry0, magic);
    else
    for (int r = 0; r < p.R; ++r) {
        const int64_t ib = r * idx_stride + entry0;
        const int64_t vb = r * val_stride + entry0;
        for (int it = 0; it < scatter_iters; ++it) {
            const uint32_t el = static_cast<uint32_t>(it * kWave + lane);
            const bool in = el < group_entries;
            const uint32_t lrow = (k == 1) ? el : __umulhi(el, magic);
            const bool chunk_start = (el - lrow * static_cast<uint32_t>(k)) == 0u;
            int at[4], addr[4];
            float v[4];
            bool ok[4];
            bool bad = false;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t e = static_cast<int64_t>(q) * group_entries + el;
                at[q] = in ? load_payload_index(idx, ib + e, p.idx_u8) : -1;
                v[q] = in ? load_payload_value(val, vb + e, p.val_dtype) : 0.0f;
                ok[q] = in && at[q] >= 0 && at[q] < S;
                addr[q] = (8 * q + static_cast<int>(lrow)) * kRow + at[q];
                const int prev = __shfl_up(at[q], 1);
                bad = bad || (in && lane > 0 && !chunk_start && prev >= at[q]);
            }
            if (__any(bad)) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ok[q]) atomicAdd(&buf[addr[q]], v[q]);
            } else {
                float a[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) a[q] = ok[q] ? buf[addr[q]] : 0.0f;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ok[q]) buf[addr[q]] = a[q] + v[q];
            }
        }
    }
    wave_lds_sync();
}

// Last phase of decompress: y (four consecutive elements of a row from get_y4(row, col)),
// optional sign, parameter update (plain or Decoupled AdamW), coalesced.  Nothing else of this
// wavefront is in flight here and the transform's registers are free, so the parameters (and
// moments) of a batch of iterations are requested at once before any of them is used: with one
// wavefront per SIMD every separate wait costs a full memory latency.
template <int NB, bool PARAM_BF16, class GetY>
__device__ __forceinline__ void update_params_rows(const KParams& p, int lane, int64_t base,
                                                   void* __restrict__ params, const AdamPtrs& ad,
                                                   float* __restrict__ presign_dbg, GetY get_y4) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S;
    constexpr int kBatch = (G::kVecIters % 8 == 0) ? 8 : 4;
    static_assert(G::kVecIters % kBatch == 0, "whole batches");
#pragma unroll 1
    for (int b = 0; b < G::kVecIters; b += kBatch) {
        float4 old4[kBatch], m4[kBatch], v4[kBatch], x4[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int64_t i = base + 4 * (lane + kWave * (b + j));
            if constexpr (PARAM_BF16) {
                const uint2 pb = ld_u2<false>(static_cast<const uint16_t*>(params) + i);
                old4[j] = make_float4(__uint_as_float(pb.x << 16),
                                      __uint_as_float(pb.x & 0xFFFF0000u),
                                      __uint_as_float(pb.y << 16),
                                      __uint_as_float(pb.y & 0xFFFF0000u));
            } else {
                old4[j] = ld_f4<false>(static_cast<const float*>(params) + i);
            }
            x4[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (p.adam) {
                m4[j] = ld_f4<false>(ad.m + i);
                v4[j] = ld_f4<false>(ad.v + i);
                if (p.amsgrad) x4[j] = ld_f4<false>(ad.vmax + i);
            }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int e4 = 4 * (lane + kWave * (b + j));
            const int row = e4 / S, col = e4 - row * S;
            const int64_t i = base + e4;
            const float4 y4 = get_y4(row, col);
            if (presign_dbg) st_f4<false>(presign_dbg + i, y4);
            const float y[4] = {y4.x, y4.y, y4.z, y4.w};
            const float old[4] = {old4[j].x, old4[j].y, old4[j].z, old4[j].w};
            float nw[4];
            if (p.adam) {
                float m[4] = {m4[j].x, m4[j].y, m4[j].z, m4[j].w};
                float v[4] = {v4[j].x, v4[j].y, v4[j].z, v4[j].w};
                float x[4] = {x4[j].x, x4[j].y, x4[j].z, x4[j].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    nw[c] = adamw_step(p, old[c], sign_or_self(y[c], p.use_sign), m[c], v[c], x[c]);
                st_f4<false>(ad.m + i, make_float4(m[0], m[1], m[2], m[3]));
                st_f4<false>(ad.v + i, make_float4(v[0], v[1], v[2], v[3]));
                if (p.amsgrad) st_f4<false>(ad.vmax + i, make_float4(x[0], x[1], x[2], x[3]));
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    nw[c] = fmaf(-p.lr, sign_or_self(y[c], p.use_sign), old[c] * p.wd_scale);
            }
            if constexpr (PARAM_BF16) {
                uint2 o;
                o.x = pack_bf16x2(nw[0], nw[1]);
                o.y = pack_bf16x2(nw[2], nw[3]);
                *reinterpret_cast<uint2*>(static_cast<uint16_t*>(params) + i) = o;
            } else {
                st_f4<false>(static_cast<float*>(params) + i,
                             make_float4(nw[0], nw[1], nw[2], nw[3]));
            }
        }
    }
}

// Decompress-and-update half on full tiles of 32 chunks (transmitted indices, DCT domain).
template <int NB, bool PARAM_BF16>
__global__ __launch_bounds__(kWave)
__attribute__((amdgpu_waves_per_eu(MfmaGeom<NB>::kWavesPerSimd))) void decompress_mfma(
    KParams p, int64_t tiles, int vec_scatter, const void* __restrict__ idx, int64_t idx_stride,
    const void* __restrict__ val, int64_t val_stride, void* __restrict__ params, AdamPtrs ad,
    float* __restrict__ presign_dbg) {
    using G = MfmaGeom<NB>;
    constexpr int S = G::S, kRow = G::kRow, W = G::kTab;
    __shared__ __attribute__((aligned(16))) float buf[kMfmaChunks * kRow];
    __shared__ float tab[W];

    const int lane = threadIdx.x;
    const int t = lane & 31, h = lane >> 5;
    const int k = p.k;
    build_cos_table_quarter<S>(tab, lane);
    // entry -> chunk within a group of 8 chunks: floor(e / k) = umulhi(e, ceil(2^32 / k)),
    // exact for e < 8*256
    const uint32_t magic = entry_magic(k);
    const float out_scale = p.alpha * p.inv_R;
    const float row0_fix = (p.alpha0 - p.alpha) * p.inv_R;
    wave_lds_sync();

    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t base = tile * static_cast<int64_t>(kMfmaChunks * S);
        const int64_t entry0 = tile * static_cast<int64_t>(kMfmaChunks) * k;

        scatter_tile<NB>(buf, p, lane, vec_scatter, idx, idx_stride, val, val_stride, entry0, magic);
        wave_lds_sync();

        // ---- y^T = D^T * (alpha_j a_j / R)^T; the scale is applied to the result:
        // y = (alpha/R) * sum_j a_j cos(..) + ((alpha0 - alpha)/R) * a_0
        const float fix = row0_fix * buf[t * kRow];
        inverse_to_lds<NB>(buf, tab, t, h,
                           [out_scale, fix](float y) { return fmaf(y, out_scale, fix); });
        wave_lds_sync();

        // ---- sign and parameter update, coalesced
        update_params_rows<NB, PARAM_BF16>(p, lane, base, params, ad, presign_dbg,
                                           [&](int row, int col) {
                                               return *reinterpret_cast<const float4*>(
                                                   &buf[row * kRow + col]);
                                           });
        wave_lds_sync();
    }
}

}  // namespace deto
