// Two lanes per chunk: kernels for the chunk sizes whose coefficients do not fit one lane
// (96, 128, 192 and 256 of the paper's Appendix B sweep; decompress: 192 and 256), top-k
// selection with transmitted indices.  They take what the wavefront-per-class kernels
// (split_kernels.hip.h) do not: the narrow payload formats and k > S/2.
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
// Selection: each lane sorts its magnitudes, the two sorted lists meet in LDS (see
// compress_pair).  Emission: each lane knows the partner's kept set as a bit mask.
#pragma once

#include "fast_dct.hip.h"
#include "mfma_kernels.hip.h"
#include "sort_network.hip.h"

namespace deto {

template <int S>
struct PairGeom {
    static_assert(S % 32 == 0, "two lanes, halves in 16-byte pieces, 32-row tiles");
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

// Forward: v = the lane's folded half; out: c[m] = alpha_j * coefficient 2m + h.
// (Running the SAME DCT-II on both lanes, the odd lane with its input multiplied by
// 2 cos(pi (2n+1) / (4H)) and a running difference O[k] = V[k] - O[k-1] on the output, would
// avoid the two code paths; its transpose for the inverse measured 1.1e-5 of the chunk scale
// at H = 128, beyond the parity tolerance, so both directions keep the plane-rotation DCT-IV.)
template <int H>
__device__ __forceinline__ void forward_half(int h, float alpha0, float alpha, float (&c)[H]) {
    if (h == 0) FastDct<H>::dct2(c);
    else FastDct<H>::dct4(c);
    c[0] *= h ? alpha : alpha0;      // coefficient 0 is lane 0's c[0]
#pragma unroll
    for (int m = 1; m < H; ++m) c[m] *= alpha;
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

// 2*word + (mag >= thr): a compare into the carry and an add with carry
__device__ __forceinline__ uint32_t push_at_least(uint32_t word, uint32_t mag, uint32_t thr) {
    asm("v_cmp_ge_u32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
        : "+v"(word)
        : "v"(mag), "v"(thr)
        : "vcc");
    return word;
}

// Compress half on full tiles of 32 chunks (top-k selection, DCT domain).
//
// Selection.  Each lane sorts the magnitudes of its H coefficients in registers (sorting
// network), the two sorted lists of a chunk meet in the chunk's LDS row (free by then), and
// the k-th largest of their union follows from a binary search over how many of the k come
// from the first list (7 steps of two LDS reads for H = 64) instead of a search over the 31
// magnitude bits with a count over all coefficients per step.  Works for any k at run time.
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
    // payload staging inside a chunk's row: values at row[pos], indices at row[kIdx0 + pos];
    // what a lane drops goes to a dump slot of its own past the tile (and kIdx0 floats on)
    constexpr int kIdx0 = H + 4;
    constexpr int kTile = kMfmaChunks * kRow;
    __shared__ __attribute__((aligned(16))) float buf[kTile + kWave + kIdx0];

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
    const int64_t base = tile * static_cast<int64_t>(kMfmaChunks * S);
    const int64_t chunk0 = tile * kMfmaChunks;
    float* row = &buf[t * kRow];

    fold_tile_rows<NB, GRAD_BF16>(buf, p, lane, grad, mom, base);
    wave_lds_sync();

    // ---- the lane's coefficients c[m] = coefficient 2m + h of chunk t
    float c[H];
    fold_halves<S>(row, h, c);
    forward_half<H>(h, p.alpha0, p.alpha, c);
    if (coeff_dbg) {
        float* dbg = coeff_dbg + (chunk0 + t) * S + h;
#pragma unroll
        for (int m = 0; m < H; ++m) dbg[2 * m] = c[m];
    }

    // ---- k-th largest magnitude T of chunk t
    uint32_t T;
    {
        uint32_t a[H];
#pragma unroll
        for (int m = 0; m < H; ++m) a[m] = __float_as_uint(c[m]) & 0x7FFFFFFFu;
        sort_desc<H>(a);
        wave_lds_sync();
        uint32_t* lst = reinterpret_cast<uint32_t*>(row) + h * H;
#pragma unroll
        for (int q = 0; q < H / 4; ++q)
            *reinterpret_cast<uint4*>(lst + 4 * q) =
                make_uint4(a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]);
        wave_lds_sync();
        // i of the k largest come from list 0 and k - i from list 1: the smallest i for which
        // list0[i] (first one left out) does not exceed list1[k-i-1] (last one taken)
        const uint32_t* l0 = reinterpret_cast<const uint32_t*>(row);
        const uint32_t* l1 = l0 + H;
        int lo = k > H ? k - H : 0, hi = k < H ? k : H;
        constexpr int kSteps = H <= 63 ? 6 : (H <= 127 ? 7 : 8);   // ceil(log2(H + 1))
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
        T = min(n0 > 0 ? t0 : 0xFFFFFFFFu, n1 > 0 ? t1 : 0xFFFFFFFFu);
    }

    // ---- kept set of this lane (bit m) and of the partner: magnitude >= T, unless more than k
    // magnitudes reach T (a tie at the threshold): then only those above T, and the chunk
    // goes through the whole-wavefront pass that adds the lowest indices among the equals
    uint32_t own[NW], other[NW];
    auto mark = [&](uint32_t thr) -> int {
#pragma unroll
        for (int w = 0; w < NW; ++w) own[w] = 0u;
        static_for<0, H>([&](auto I) {
            constexpr int m = H - 1 - I;   // descending so that shifting lands bit m at m
            // own = 2*own + (|c[m]| >= thr): a compare into the carry and an add with carry
            own[m / 32] = push_at_least(own[m / 32], __float_as_uint(c[m]) & 0x7FFFFFFFu, thr);
        });
        int cnt = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) cnt += __popc(own[w]);
        return cnt + __shfl_xor(cnt, 32);
    };
    uint32_t thr_gt = T, thr_eq = 0xFFFFFFFFu;
    int need = 0;
    {
        const int cnt = mark(T);
        const bool tie = cnt != k;
        if (__any(tie)) {
            if (tie) {
                thr_gt = T + 1u;     // <= 0x80000000: no magnitude reaches that
                thr_eq = T;
            }
            const int above = mark(thr_gt);
            if (tie) need = k - above;
        }
    }
#pragma unroll
    for (int w = 0; w < NW; ++w)
        other[w] = static_cast<uint32_t>(__shfl_xor(static_cast<int>(own[w]), 32));

    // ---- chunks with ties take the whole-wavefront pass over the LDS row; their lanes park
    // the coefficients there and read the remainder back
    const uint64_t tie_lanes = __ballot(need != 0);
    wave_lds_sync();
    if (tie_lanes) {
#pragma unroll
        for (int m = 0; m < H; ++m) row[2 * m + h] = c[m];
        wave_lds_sync();
        emit_tied_chunks<NB>(buf, p, lane, need, thr_gt, thr_eq, chunk0, idx_out, val_out,
                             nullptr);
        wave_lds_sync();
    }

    // ---- payload out, remainder in (settled chunks).  Lane h owns the indices 2m + h in
    // ascending order; the position of an element is its rank among the lane's kept
    // elements plus the partner's kept elements with a smaller index: m' < m for h = 0,
    // m' <= m for h = 1.  fp32 + int32 payloads with k <= S/2 are staged in the chunk's LDS row
    // and leave with coalesced stores (16 bytes per lane when k is a multiple of 4, else 4);
    // other formats are stored entry by entry.
    const bool staged = p.val_dtype == 0 && !p.idx_u8 && k <= H;
    if (need == 0 && staged) {
        // the partner's bits lined up with this lane's steps: after element m the position
        // advances by own bit m plus the partner's bit m (h = 0) or m + 1 (h = 1)
        uint32_t oth[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t up = (w + 1 < NW) ? other[w + 1] : 0u;
            oth[w] = h ? __builtin_amdgcn_alignbit(up, other[w], 1) : other[w];
        }
        char* lds = reinterpret_cast<char*>(buf);
        const uint32_t dump = static_cast<uint32_t>(sizeof(float)) * (kTile + lane);
        uint32_t at = static_cast<uint32_t>(sizeof(float)) * (t * kRow) +
                      (h ? 4u * (other[0] & 1u) : 0u);
        const float hf = __int_as_float(h);
        static_for<0, H>([&](auto m) {
            const uint32_t kb = (own[m / 32] >> (m % 32)) & 1u;
            const uint32_t ob = (oth[m / 32] >> (m % 32)) & 1u;
            const bool keep = kb != 0u;
            const uint32_t a = keep ? at : dump;
            *reinterpret_cast<float*>(lds + a) = c[m];
            *reinterpret_cast<float*>(lds + a + sizeof(float) * kIdx0) =
                __int_as_float(__float_as_int(hf) + 2 * m);
            at += 4u * kb + 4u * ob;
            c[m] = (keep ? 0.0f : c[m]) * ((m == 0 && h == 0) ? p.alpha0 : p.alpha);
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
        float* vo = static_cast<float*>(val_out) + chunk0 * k;
        int32_t* io = static_cast<int32_t*>(idx_out) + chunk0 * k;
        if (k % 4 == 0) {
            const int quads = 8 * k;                       // 16-byte pieces of the tile
            for (int q = lane; q < quads; q += kWave) {
                const uint32_t e = 4u * static_cast<uint32_t>(q);
                const uint32_t r = __umulhi(e, magic);     // chunk of the tile, k >= 4
                const uint32_t j = e - r * static_cast<uint32_t>(k);
                if ((tie_lanes >> r) & 1ull) continue;     // written by the tie pass
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
            for (uint32_t e = lane; e < static_cast<uint32_t>(kMfmaChunks * k); e += kWave) {
                const uint32_t r = (k == 1) ? e : __umulhi(e, magic);
                const uint32_t j = e - r * static_cast<uint32_t>(k);
                if ((tie_lanes >> r) & 1ull) continue;
                const float* src = &buf[r * kRow + j];
                vo[e] = src[0];
                io[e] = __float_as_int(src[kIdx0]);
            }
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
