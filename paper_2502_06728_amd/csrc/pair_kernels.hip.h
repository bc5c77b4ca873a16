// Two lanes per chunk: kernels for the chunk sizes whose coefficients do not fit one lane
// (192 and 256 of the paper's Appendix B sweep), top-k selection with transmitted indices.
//
// One wavefront (= one workgroup) owns a tile of 32 complete chunks as a 32 x S matrix in LDS
// (row = chunk), like the matrix-core kernels, but the transform is the register-resident fast
// DCT split once by hand between the two lanes t and t + 32 of chunk t (H = S/2):
//   lane h = 0 forms u_n = x_n + x_{S-1-n} and computes the even coefficients dct2_H(u),
//   lane h = 1 forms w_n = x_n - x_{S-1-n} and computes the odd  coefficients dct4_H(w)
// (the first level of the dct2 recursion of fast_dct.hip.h).  Lane h therefore owns the
// coefficients j = 2m + h, m < H, in registers.  The inverse runs the same split backwards:
// E = dct3_H(even part) on lane 0, O = dct4_H(odd part) on lane 1, and the streaming pass forms
// y_n = E_n + O_n, y_{S-1-n} = E_n - O_n from the two halves parked in the LDS row.
// Selection and payload emission follow the matrix-core kernels (binary search for the k-th
// largest magnitude with the two lanes' counts added, partner's kept set as a bit mask).
#pragma once

#include "fast_dct.hip.h"
#include "mfma_kernels.hip.h"

namespace deto {

template <int S>
struct PairGeom {
    static_assert(S % 64 == 0, "two lanes, halves in 16-byte pieces, 32-row tiles");
    static constexpr int NB = S / 32;
    static constexpr int H = S / 2;                 // coefficients per lane
    static constexpr int kRow = MfmaGeom<NB>::kRow;
    static constexpr int kWords = (H + 31) / 32;    // mask words per lane
    static constexpr size_t kSmemBytes = sizeof(float) * kMfmaChunks * kRow;
};

// v[m] = x[m] + x[S-1-m] (h = 0) or x[m] - x[S-1-m] (h = 1) from the lane's chunk row
template <int S>
__device__ __forceinline__ void fold_halves(const float* __restrict__ row, int h,
                                            float (&v)[S / 2]) {
    constexpr int H = S / 2;
    const float sgn = h ? -1.0f : 1.0f;
#pragma unroll
    for (int q = 0; q < H / 4; ++q) {
        const float4 a = *reinterpret_cast<const float4*>(row + 4 * q);
        const float4 b = *reinterpret_cast<const float4*>(row + S - 4 - 4 * q);
        v[4 * q] = fmaf(sgn, b.w, a.x);
        v[4 * q + 1] = fmaf(sgn, b.z, a.y);
        v[4 * q + 2] = fmaf(sgn, b.y, a.z);
        v[4 * q + 3] = fmaf(sgn, b.x, a.w);
    }
}

// The lane's half of the inverse: E (h = 0) or O (h = 1), parked in the row as [E | O]
template <int S>
__device__ __forceinline__ void inverse_half_to_row(float* __restrict__ row, int h,
                                                    float (&v)[S / 2]) {
    constexpr int H = S / 2;
    if (h == 0) FastDct<H>::dct3(v);
    else FastDct<H>::dct4(v);
    wave_lds_sync();
#pragma unroll
    for (int q = 0; q < H / 4; ++q)
        *reinterpret_cast<float4*>(row + h * H + 4 * q) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}

// four consecutive output elements col .. col+3 of a row holding [E | O]
template <int S>
__device__ __forceinline__ float4 combine_halves(const float* __restrict__ row, int col) {
    constexpr int H = S / 2;
    if (col < H) {
        const float4 e = *reinterpret_cast<const float4*>(row + col);
        const float4 o = *reinterpret_cast<const float4*>(row + H + col);
        return make_float4(e.x + o.x, e.y + o.y, e.z + o.z, e.w + o.w);
    }
    const int n0 = S - 4 - col;     // elements col+i are the mirror images of n0+3-i
    const float4 e = *reinterpret_cast<const float4*>(row + n0);
    const float4 o = *reinterpret_cast<const float4*>(row + H + n0);
    return make_float4(e.w - o.w, e.z - o.z, e.y - o.y, e.x - o.x);
}

// Compress half on full tiles of 32 chunks (top-k selection, DCT domain).
template <int S, bool GRAD_BF16>
__global__ __launch_bounds__(kWave) void compress_pair(KParams p, int64_t tiles, int64_t n,
                                                       int64_t n_chunks,
                                                       const void* __restrict__ grad,
                                                       float* __restrict__ mom,
                                                       void* __restrict__ idx_out,
                                                       void* __restrict__ val_out,
                                                       float* __restrict__ coeff_dbg) {
    using G = PairGeom<S>;
    constexpr int NB = G::NB, H = G::H, kRow = G::kRow, NW = G::kWords;
    __shared__ __attribute__((aligned(16))) float buf[kMfmaChunks * kRow];

    const int lane = threadIdx.x;
    const int t = lane & 31, h = lane >> 5;
    const int k = p.k;

    // One tile per workgroup.  A loop over tiles invites the compiler to hoist what does not
    // change from tile to tile (the lane's payload index constants, row addresses) out of it
    // and, with every register taken, to spill it: a scratch reload per coefficient.
    const int64_t tile = blockIdx.x;
    if (tile >= tiles) {
        // surplus workgroups: the chunks past the last full tile, one each, on the general
        // per-chunk code, side by side with the tiles instead of in a launch of their own
        static_assert(sizeof(GenericCompressSmem) <= sizeof(buf), "tail code borrows the tile");
        compress_generic_chunks<GRAD_BF16>(p, n, tiles * kMfmaChunks + (tile - tiles), n_chunks,
                                           gridDim.x - tiles,
                                           *reinterpret_cast<GenericCompressSmem*>(buf), grad, mom,
                                           idx_out, val_out, coeff_dbg);
        return;
    }
    {
        const int64_t base = tile * static_cast<int64_t>(kMfmaChunks * S);
        const int64_t chunk0 = tile * kMfmaChunks;
        float* row = &buf[t * kRow];

        fold_tile_rows<NB, GRAD_BF16>(buf, p, lane, grad, mom, base);
        wave_lds_sync();

        // ---- the lane's coefficients c[m] = coefficient 2m + h of chunk t
        float c[H];
        fold_halves<S>(row, h, c);
        if (h == 0) FastDct<H>::dct2(c);
        else FastDct<H>::dct4(c);
        c[0] *= h ? p.alpha : p.alpha0;      // coefficient 0 is lane 0's c[0]
#pragma unroll
        for (int m = 1; m < H; ++m) c[m] *= p.alpha;
        if (coeff_dbg) {
            float* dbg = coeff_dbg + (chunk0 + t) * S + h;
#pragma unroll
            for (int m = 0; m < H; ++m) dbg[2 * m] = c[m];
        }

        // ---- k-th largest magnitude of chunk t by binary search on its bits.  The signs
        // are parked in mask words meanwhile, so a count is two instructions per coefficient
        // (mag - cand is exact, its sign bit goes into a collector, one popcount per 32).
        uint32_t sgn[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) sgn[w] = 0u;
        static_for<0, H>([&](auto I) {
            constexpr int m = H - 1 - I;   // descending so that shifting lands bit m at m
            const uint32_t b = __float_as_uint(c[m]);
            sgn[m / 32] = (sgn[m / 32] << 1) | (b >> 31);
            c[m] = __uint_as_float(b & 0x7FFFFFFFu);
        });
        // the search reads every magnitude 31 times: have them in vector registers proper,
        // not in the accumulation registers the transform's temporaries spilled into
#pragma unroll
        for (int m = 0; m < H; ++m) asm volatile("" : "+v"(c[m]));
        auto count_at_least = [&](uint32_t cand) -> int {
            int below = 0;
#pragma unroll
            for (int w = 0; w < H; w += 32) {
                uint32_t coll = 0u;
#pragma unroll
                for (int i = 0; i < 32 && w + i < H; ++i)
                    coll = __builtin_amdgcn_alignbit(coll, __float_as_uint(c[w + i]) - cand, 31);
                below += __popc(coll);
            }
            const int own = H - below;
            return own + __shfl_xor(own, 32);
        };
        uint32_t T = 0u, thr_gt = 0u;
        bool done = false;
#pragma unroll 1
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
            const uint32_t gt = T + 1u;                       // <= 0x80000000: nothing reaches it
            const int cg_all = count_at_least(gt & 0x7FFFFFFFu);   // every lane takes part
            if (!done) {
                thr_gt = gt;
                thr_eq = T;
                need = k - ((gt > 0x7FFFFFFFu) ? 0 : cg_all);
            }
        }
        // kept set of this lane (bit m), and the partner's
        uint32_t own[NW], other[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) own[w] = 0u;
        static_for<0, H>([&](auto I) {
            constexpr int m = H - 1 - I;
            own[m / 32] = (own[m / 32] << 1) | (__float_as_uint(c[m]) >= thr_gt ? 1u : 0u);
        });
#pragma unroll
        for (int w = 0; w < NW; ++w)
            other[w] = static_cast<uint32_t>(__shfl_xor(static_cast<int>(own[w]), 32));
        // signs back
        static_for<0, H>([&](auto m) {
            c[m] = __uint_as_float(__float_as_uint(c[m]) | (((sgn[m / 32] >> (m % 32)) & 1u) << 31));
        });

        // ---- chunks with ties at the k-th magnitude take the whole-wavefront pass over the
        // LDS row; their lanes park the coefficients there and read the remainder back
        const uint64_t tie_lanes = __ballot(need != 0);
        if (tie_lanes) {
            wave_lds_sync();
#pragma unroll
            for (int m = 0; m < H; ++m) row[2 * m + h] = c[m];
            wave_lds_sync();
            emit_tied_chunks<NB>(buf, p, lane, need, thr_gt, thr_eq, chunk0, idx_out, val_out,
                                 nullptr);
        }
        wave_lds_sync();

        // ---- payload out, remainder in (settled chunks).  Lane h owns the indices 2m + h in
        // ascending order; the position of an element is its rank among the lane's kept
        // elements plus the partner's kept elements with a smaller index: m' < m for h = 0,
        // m' <= m for h = 1.  The chunk's LDS row is free by now (its contents live in the two
        // lanes' registers), so fp32 + int32 payloads with k a multiple of 4 and k <= S/2 are
        // staged there, values at row[pos] and indices at row[S/2 + pos], and leave with
        // 16-byte coalesced stores; a scattered 4-byte store instruction per coefficient costs
        // several times more.  Other formats are stored entry by entry.
        const bool staged = p.val_dtype == 0 && !p.idx_u8 && (k % 4) == 0 && k <= H;
        if (need == 0 && staged) {
            // branch-free: a dropped element is written to the row's padding slots instead
            int pos = 0;
            static_for<0, H>([&](auto m) {
                const uint32_t pbit = (other[m / 32] >> (m % 32)) & 1u;
                const bool keep = (own[m / 32] >> (m % 32)) & 1u;
                if (h) pos += static_cast<int>(pbit);
                const bool put = keep && pos < k;
                row[put ? pos : S] = c[m];
                row[put ? H + pos : S + 1] = __int_as_float(2 * m + h);
                pos += keep ? 1 : 0;
                if (!h) pos += static_cast<int>(pbit);
                c[m] = (put ? 0.0f : c[m]) * ((m == 0 && h == 0) ? p.alpha0 : p.alpha);
            });
        } else if (need == 0) {
            const int64_t cbase = (chunk0 + t) * k;
            int pos = 0;
            static_for<0, H>([&](auto m) {
                const uint32_t pbit = (other[m / 32] >> (m % 32)) & 1u;
                const bool keep = (own[m / 32] >> (m % 32)) & 1u;
                if (h) pos += static_cast<int>(pbit);
                float rem = c[m];
                if (keep && pos < k) {
                    store_payload_index(idx_out, cbase + pos, p.idx_u8, 2 * m + h);
                    store_payload_value(val_out, cbase + pos, p.val_dtype, c[m]);
                    rem = c[m] - payload_roundtrip(p.val_dtype, c[m]);
                }
                pos += keep ? 1 : 0;
                if (!h) pos += static_cast<int>(pbit);
                c[m] = rem * ((m == 0 && h == 0) ? p.alpha0 : p.alpha);
            });
        } else {
#pragma unroll
            for (int m = 0; m < H; ++m) c[m] = row[2 * m + h];   // alpha_j * remainder
        }
        wave_lds_sync();
        if (staged) {
            // the tile's 32*k entries are contiguous in both payload arrays
            const uint32_t magic = entry_magic(k);
            const int quads = 8 * k;                       // 16-byte pieces of the tile
            float* vo = static_cast<float*>(val_out) + chunk0 * k;
            int32_t* io = static_cast<int32_t*>(idx_out) + chunk0 * k;
            for (int q = lane; q < quads; q += kWave) {
                const uint32_t e = 4u * static_cast<uint32_t>(q);
                const uint32_t r = __umulhi(e, magic);     // chunk of the tile, k >= 4
                const uint32_t j = e - r * static_cast<uint32_t>(k);
                if ((tie_lanes >> r) & 1ull) continue;     // written by the tie pass
                const float* src = &buf[r * kRow + j];
                st_f4<false>(vo + e, *reinterpret_cast<const float4*>(src));
                const float4 iv = *reinterpret_cast<const float4*>(src + H);
                *reinterpret_cast<int4*>(io + e) =
                    make_int4(__float_as_int(iv.x), __float_as_int(iv.y), __float_as_int(iv.z),
                              __float_as_int(iv.w));
            }
            wave_lds_sync();
        }

        // ---- new momentum = inverse transform of the remainder
        inverse_half_to_row<S>(row, h, c);
        wave_lds_sync();
        {
            using MG = MfmaGeom<NB>;
#pragma unroll 4
            for (int it = 0; it < MG::kVecIters; ++it) {
                const int e4 = 4 * (lane + kWave * it);
                const int r = e4 / S, col = e4 - r * S;
                st_f4<false>(mom + base + e4, combine_halves<S>(&buf[r * kRow], col));
            }
        }
        wave_lds_sync();
    }
}

// Decompress-and-update half on full tiles of 32 chunks (transmitted indices, DCT domain).
template <int S, bool PARAM_BF16>
__global__ __launch_bounds__(kWave) void decompress_pair(
    KParams p, int64_t tiles, int64_t n, int64_t n_chunks, int vec_scatter,
    const void* __restrict__ idx, int64_t idx_stride, const void* __restrict__ val,
    int64_t val_stride, void* __restrict__ params, AdamPtrs ad, float* __restrict__ presign_dbg) {
    using G = PairGeom<S>;
    constexpr int NB = G::NB, H = G::H, kRow = G::kRow;
    __shared__ __attribute__((aligned(16))) float buf[kMfmaChunks * kRow];

    const int lane = threadIdx.x;
    const int t = lane & 31, h = lane >> 5;
    const int k = p.k;
    const uint32_t magic = entry_magic(k);
    const float scale = p.alpha * p.inv_R, scale0 = p.alpha0 * p.inv_R;

    // One tile per workgroup.  A loop over tiles invites the compiler to hoist what does not
    // change from tile to tile (the lane's payload index constants, row addresses) out of it
    // and, with every register taken, to spill it: a scratch reload per coefficient.
    const int64_t tile = blockIdx.x;
    if (tile >= tiles) {
        static_assert(sizeof(GenericDecompressSmem) <= sizeof(buf), "tail code borrows the tile");
        decompress_generic_chunks<PARAM_BF16>(p, n, tiles * kMfmaChunks + (tile - tiles), n_chunks,
                                              gridDim.x - tiles,
                                              *reinterpret_cast<GenericDecompressSmem*>(buf), idx,
                                              idx_stride, val, val_stride, params, ad,
                                              presign_dbg);
        return;
    }
    {
        const int64_t base = tile * static_cast<int64_t>(kMfmaChunks * S);
        const int64_t entry0 = tile * static_cast<int64_t>(kMfmaChunks) * k;
        float* row = &buf[t * kRow];

        scatter_tile<NB>(buf, p, lane, vec_scatter, idx, idx_stride, val, val_stride, entry0, magic);
        wave_lds_sync();

        // ---- the lane's half of the accumulated coefficients: a[2m + h] * alpha_j / R
        float v[H];
#pragma unroll
        for (int q = 0; q < S / 4; ++q) {
            const float4 a = *reinterpret_cast<const float4*>(row + 4 * q);
            v[2 * q] = (h ? a.y : a.x) * scale;
            v[2 * q + 1] = (h ? a.w : a.z) * scale;
        }
        if (h == 0) v[0] = row[0] * scale0;
        inverse_half_to_row<S>(row, h, v);
        wave_lds_sync();

        update_params_rows<NB, PARAM_BF16>(p, lane, base, params, ad, presign_dbg,
                                           [&](int r, int col) {
                                               return combine_halves<S>(&buf[r * kRow], col);
                                           });
        wave_lds_sync();
    }
}

}  // namespace deto
