// Tiled kernels for power-of-two chunk sizes: the bandwidth path.
//
// Mapping.  A workgroup is ONE wavefront and owns a tile of 64 consecutive chunks.
//   phase 1  all 64 lanes stream the tile from HBM with 16-byte accesses (fully
//            coalesced), do the element-wise part there, and park the tile in LDS;
//   phase 2  lane L picks up chunk L of the tile (one LDS row) into registers: the DCT,
//            the selection and the inverse DCT of that chunk are private VALU work of one
//            lane, with no cross-lane traffic and no divergence (fast_dct.hip.h);
//   phase 3  results go back through LDS and leave with 16-byte coalesced stores.
// LDS rows are padded by 16 bytes so both the coalesced phase (consecutive lanes ->
// consecutive 16 B) and the row phase (lane L -> row L) are free of bank conflicts.
//
// Selection (top-k, ties to the lower index): the magnitudes' bit patterns are sorted as
// two halves with a Batcher odd-even merge network in registers; the k-th largest
// magnitude T follows from the two sorted halves as max_i min(A[i-1], B[k-i-1]); entries
// with magnitude >= T are kept.  Only if some chunk of the wavefront has a tie AT the
// threshold does the wavefront take the exact path that keeps the lowest indices.
// Striding keeps a fixed bit pattern, Random builds each chunk's pattern with a
// Fisher-Yates shuffle private to the chunk's lane.
//
// Tail.  The chunks that do not fill a last tile (and a ragged last chunk) are handled in the
// same launch: the grid has one surplus workgroup per tail chunk, and those run the general
// per-chunk code (generic_kernels.hip.h) side by side with the tiles.
#pragma once

#include "deto_device.hip.h"
#include "fast_dct.hip.h"
#include "generic_kernels.hip.h"
#include "sort_network.hip.h"

namespace deto {

// K-th largest of the union of two descending arrays of length H.
template <int H, int K>
__device__ __forceinline__ uint32_t kth_largest(const uint32_t (&A)[H], const uint32_t (&B)[H]) {
    constexpr int lo = (K - H) > 0 ? (K - H) : 0;
    constexpr int hi = K < H ? K : H;
    uint32_t best = 0u;
    static_for<lo, hi + 1>([&](auto I) {
        constexpr int i = I;       // i entries from A, K - i from B
        uint32_t term;
        if constexpr (i == 0) term = B[K - 1];
        else if constexpr (i == K) term = A[K - 1];
        else term = min(A[i - 1], B[K - i - 1]);
        best = max(best, term);
    });
    return best;
}

template <int S>
struct TileGeom {
    static constexpr int kRow = S + 4;           // floats per LDS row (16 B of padding)
    static constexpr int kFloats = kWave * kRow;
    static constexpr int kElems = kWave * S;     // elements per tile
    static constexpr int kPermStride = S + 4;    // bytes per lane of Fisher-Yates scratch
    // a chunk lives in S VGPRs of its lane: 2 wavefronts per SIMD up to S = 64, 1 beyond
    static constexpr int kWavesPerSimd = S <= 64 ? 2 : 1;
    // LDS of a workgroup: the tile, or the general code's working set in a tail workgroup
    static constexpr size_t kTileBytes = sizeof(float) * kFloats;
    static constexpr size_t kCompressBytes =
        kTileBytes > sizeof(GenericCompressSmem) ? kTileBytes : sizeof(GenericCompressSmem);
    static constexpr size_t kDecompressBytes =
        kTileBytes > sizeof(GenericDecompressSmem) ? kTileBytes : sizeof(GenericDecompressSmem);
};

// Where a launch's tail lives: tiles [0, n_tiles) are full; chunks [64*n_tiles, n_chunks) go
// one per surplus workgroup to the general code.
struct TailRange {
    int64_t n;          // shard length
    int64_t n_chunks;   // ceil(n / s)
};

// A chunk's kept positions as a bit pattern: bit i%32 of word i/32 = element i is kept.
template <int S>
struct ChunkMask {
    static constexpr int kWords = (S + 31) / 32;
    uint32_t w[kWords];
    __device__ __forceinline__ uint32_t bit(int i) const { return (w[i / 32] >> (i % 32)) & 1u; }
    __device__ __forceinline__ int count() const {
        int c = 0;
#pragma unroll
        for (int j = 0; j < kWords; ++j) c += __popc(w[j]);
        return c;
    }
};

// Striding's pattern is the same for every chunk: computed on the host, passed by value.
struct MaskWords {
    uint32_t w[4];
};

template <int S>
__device__ __forceinline__ ChunkMask<S> mask_from_words(const MaskWords& m) {
    ChunkMask<S> r;
#pragma unroll
    for (int j = 0; j < ChunkMask<S>::kWords; ++j) r.w[j] = m.w[j];
    return r;
}

// ---- phase 1 of compress: m1 = beta*m + g, coalesced, into the LDS tile
template <int S, bool GRAD_BF16>
__device__ __forceinline__ void fold_tile_to_lds(const KParams& p, const void* __restrict__ grad,
                                                 const float* __restrict__ mom, int64_t ebase,
                                                 float* tile, int lane) {
    using G = TileGeom<S>;
#pragma unroll
    for (int it = 0; it < S / 8; ++it) {
        const int pe = it * 512 + lane * 8;
        const float4 ma = ld_f4<DETO_NT_COMPRESS_MOM>(mom + ebase + pe);
        const float4 mb = ld_f4<DETO_NT_COMPRESS_MOM>(mom + ebase + pe + 4);
        float g[8];
        if constexpr (GRAD_BF16) {
            const uint4 raw =
                ld_u4<DETO_NT_COMPRESS_GRAD>(static_cast<const uint16_t*>(grad) + ebase + pe);
            g[0] = __uint_as_float(raw.x << 16);
            g[1] = __uint_as_float(raw.x & 0xFFFF0000u);
            g[2] = __uint_as_float(raw.y << 16);
            g[3] = __uint_as_float(raw.y & 0xFFFF0000u);
            g[4] = __uint_as_float(raw.z << 16);
            g[5] = __uint_as_float(raw.z & 0xFFFF0000u);
            g[6] = __uint_as_float(raw.w << 16);
            g[7] = __uint_as_float(raw.w & 0xFFFF0000u);
        } else {
            const float4 ga =
                ld_f4<DETO_NT_COMPRESS_GRAD>(static_cast<const float*>(grad) + ebase + pe);
            const float4 gb =
                ld_f4<DETO_NT_COMPRESS_GRAD>(static_cast<const float*>(grad) + ebase + pe + 4);
            g[0] = ga.x; g[1] = ga.y; g[2] = ga.z; g[3] = ga.w;
            g[4] = gb.x; g[5] = gb.y; g[6] = gb.z; g[7] = gb.w;
        }
        float4 fa, fb;
        fa.x = fmaf(p.beta, ma.x, g[0]);
        fa.y = fmaf(p.beta, ma.y, g[1]);
        fa.z = fmaf(p.beta, ma.z, g[2]);
        fa.w = fmaf(p.beta, ma.w, g[3]);
        fb.x = fmaf(p.beta, mb.x, g[4]);
        fb.y = fmaf(p.beta, mb.y, g[5]);
        fb.z = fmaf(p.beta, mb.z, g[6]);
        fb.w = fmaf(p.beta, mb.w, g[7]);
        float* dst = tile + (pe / S) * G::kRow + (pe % S);
        *reinterpret_cast<float4*>(dst) = fa;
        *reinterpret_cast<float4*>(dst + 4) = fb;
    }
}

template <int S>
__device__ __forceinline__ void row_to_regs(const float* row, float (&x)[S]) {
#pragma unroll
    for (int j = 0; j < S / 4; ++j) {
        const float4 v = *reinterpret_cast<const float4*>(row + 4 * j);
        x[4 * j] = v.x; x[4 * j + 1] = v.y; x[4 * j + 2] = v.z; x[4 * j + 3] = v.w;
    }
}

template <int S>
__device__ __forceinline__ void regs_to_row(float* row, const float (&x)[S]) {
#pragma unroll
    for (int j = 0; j < S / 4; ++j)
        *reinterpret_cast<float4*>(row + 4 * j) =
            make_float4(x[4 * j], x[4 * j + 1], x[4 * j + 2], x[4 * j + 3]);
}

// debug export of one chunk's S values straight from the lane that owns the chunk
template <int S>
__device__ __forceinline__ void regs_to_global(float* dst, const float (&x)[S]) {
#pragma unroll
    for (int j = 0; j < S / 4; ++j)
        *reinterpret_cast<float4*>(dst + 4 * j) =
            make_float4(x[4 * j], x[4 * j + 1], x[4 * j + 2], x[4 * j + 3]);
}

// Length in floats of a chunk's row in the [chunk][k] staging block of the payload: room for
// k entries plus a spare slot, a multiple of 4 when k is one (the block leaves with 16-byte
// reads), and then an odd multiple of 4: the 64 lanes' rows start in 16 different groups of four
// LDS banks instead of 4 or 8 (k = 12 or 4), which would pile the lanes' scalar writes onto a
// few banks.
constexpr int staging_row(int k) {
    int pr = k + 4;
    if (k % 4 == 0 && (pr / 4) % 2 == 0) pr += 4;
    return pr;
}

// ---- phase 3a of compress: compact the kept (index, value) pairs of each chunk, ascending,
// and store the tile's payload coalesced.  The tile must be free (every lane holds its row
// in registers).  Every element is written at the running position, which only advances
// past kept ones, so a dropped element is overwritten by the next kept one.
// VAL selects the payload format: 0 = fp32 values + int32 indices; 1 (bf16) / 2 (fp16) =
// 16-bit values + byte indices (the values in c are then already rounded to that format).
template <int S, int K, int VAL = 0>
__device__ __forceinline__ void compact_and_store_payload(const float (&c)[S],
                                                          const ChunkMask<S>& mk, float* tile,
                                                          int lane,
                                                          void* __restrict__ idx_out_v,
                                                          void* __restrict__ val_out_v,
                                                          int64_t pbase) {
    using G = TileGeom<S>;
    constexpr int PR = staging_row(K);              // staging row, one spare slot + pad
    float* vrow = tile + lane * PR;
    uint8_t* ibytes = reinterpret_cast<uint8_t*>(tile + kWave * PR);   // indices as bytes
    uint8_t* irow = ibytes + lane * PR;
    static_assert(kWave * PR * 5 <= G::kFloats * 4, "staging must fit in the tile");
    {
        int pos = 0;
        static_for<0, S>([&](auto i) {
            vrow[pos] = c[i];
            irow[pos] = static_cast<uint8_t>(i);
            pos += static_cast<int>(mk.bit(i));
        });
    }
    wave_lds_sync();
    if constexpr (VAL != 0) {
        uint8_t* idx8 = static_cast<uint8_t*>(idx_out_v);
        if constexpr (VAL == 3) {
            // ternary: the lane packs the signs of its chunk's K staged values, two bits each
            // (0 = zero, 1 = +1, 3 = -1), into ceil(K/16) words
            constexpr int W = (K + 15) / 16;
            uint32_t* words = static_cast<uint32_t*>(val_out_v) + (pbase / K) * W + lane * W;
            uint32_t wv[W];
#pragma unroll
            for (int w = 0; w < W; ++w) wv[w] = 0u;
            auto put = [&](int j, float v) {
                const int b = __float_as_int(v);
                const uint32_t code =
                    b > 0 ? 1u : (static_cast<uint32_t>(b) > 0x80000000u ? 3u : 0u);
                wv[j / 16] |= code << (2 * (j % 16));
            };
            if constexpr (K % 4 == 0) {
#pragma unroll
                for (int q = 0; q < K / 4; ++q) {
                    const float4 v = *reinterpret_cast<const float4*>(vrow + 4 * q);
                    put(4 * q, v.x); put(4 * q + 1, v.y); put(4 * q + 2, v.z); put(4 * q + 3, v.w);
                }
            } else {
#pragma unroll
                for (int j = 0; j < K; ++j) put(j, vrow[j]);
            }
            if constexpr (W == 2) *reinterpret_cast<uint2*>(words) = make_uint2(wv[0], wv[1]);
            else {
#pragma unroll
                for (int w = 0; w < W; ++w) words[w] = wv[w];
            }
        } else if constexpr (K % 4 == 0) {
            // 16-bit values, four entries per lane and store
            uint16_t* val16 = static_cast<uint16_t*>(val_out_v);
#pragma unroll
            for (int it = 0; it < K / 4; ++it) {
                const int e = it * 256 + lane * 4;
                const int r = e / K, col = e % K;
                const float4 v = *reinterpret_cast<const float4*>(tile + r * PR + col);
                uint2 packed;
                if constexpr (VAL == 1) {
                    packed.x = pack_bf16x2(v.x, v.y);
                    packed.y = pack_bf16x2(v.z, v.w);
                } else {
                    packed.x =
                        encode16<VAL>(v.x) | (static_cast<uint32_t>(encode16<VAL>(v.y)) << 16);
                    packed.y =
                        encode16<VAL>(v.z) | (static_cast<uint32_t>(encode16<VAL>(v.w)) << 16);
                }
                *reinterpret_cast<uint2*>(val16 + pbase + e) = packed;
            }
        } else {
            // k = 1, 2: the lane stores its own chunk's entries
            uint16_t* val16 = static_cast<uint16_t*>(val_out_v) + pbase + lane * K;
#pragma unroll
            for (int j = 0; j < K; ++j) val16[j] = encode16<VAL>(vrow[j]);
        }
        // byte indices
        if (idx8) {
            if constexpr (K % 4 == 0) {
#pragma unroll
                for (int it = 0; it < K / 4; ++it) {
                    const int e = it * 256 + lane * 4;
                    const int r = e / K, col = e % K;
                    *reinterpret_cast<uint32_t*>(idx8 + pbase + e) =
                        *reinterpret_cast<const uint32_t*>(ibytes + r * PR + col);
                }
            } else {
#pragma unroll
                for (int j = 0; j < K; ++j) idx8[pbase + lane * K + j] = irow[j];
            }
        }
        wave_lds_sync();
        return;
    }
    int32_t* idx_out = static_cast<int32_t*>(idx_out_v);
    float* val_out = static_cast<float*>(val_out_v);
    if constexpr (K % 4 == 0) {
#pragma unroll
        for (int it = 0; it < K / 4; ++it) {
            const int e = it * 256 + lane * 4;
            const int r = e / K, col = e % K;
            st_f4<DETO_NT_COMPRESS_PAYLOAD>(val_out + pbase + e,
                                            *reinterpret_cast<const float4*>(tile + r * PR + col));
            if (idx_out) {
                const uint32_t pk = *reinterpret_cast<const uint32_t*>(ibytes + r * PR + col);
                st_u4<DETO_NT_COMPRESS_PAYLOAD>(
                    idx_out + pbase + e,
                    make_uint4(pk & 0xFFu, (pk >> 8) & 0xFFu, (pk >> 16) & 0xFFu, pk >> 24));
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < K; ++j) {
            val_out[pbase + lane * K + j] = vrow[j];
            if (idx_out) idx_out[pbase + lane * K + j] = irow[j];
        }
    }
    wave_lds_sync();
}

// ---- phase 3b of compress: the tile (rows = residual momentum) out, coalesced
template <int S>
__device__ __forceinline__ void store_tile_momentum(const float* tile, float* __restrict__ mom,
                                                    int64_t ebase, int lane) {
    using G = TileGeom<S>;
#pragma unroll
    for (int it = 0; it < S / 8; ++it) {
        const int pe = it * 512 + lane * 8;
        const float* src = tile + (pe / S) * G::kRow + (pe % S);
        st_f4<DETO_NT_COMPRESS_MOM_ST>(mom + ebase + pe, *reinterpret_cast<const float4*>(src));
        st_f4<DETO_NT_COMPRESS_MOM_ST>(mom + ebase + pe + 4,
                                       *reinterpret_cast<const float4*>(src + 4));
    }
}

// Random scheme: the kept positions of one chunk as a bit mask.  `perm` is S bytes of LDS
// private to the calling lane.  Only perm[t] needs writing back: place j is never read
// again once step j has taken its value.
template <int S, int K>
__device__ __forceinline__ ChunkMask<S> random_mask(uint64_t seed, uint64_t step, uint64_t chunk,
                                                    uint8_t* perm) {
#pragma unroll
    for (int w = 0; w < S / 4; ++w)
        reinterpret_cast<uint32_t*>(perm)[w] = 0x03020100u + 0x04040404u * w;
    const uint64_t key = chunk_key(seed, step, chunk);
    ChunkMask<S> mask;
#pragma unroll
    for (int w = 0; w < ChunkMask<S>::kWords; ++w) mask.w[w] = 0u;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int t = j + static_cast<int>(bounded(draw(key, j), S - j));
        const uint8_t pj = perm[j];
        const uint8_t pt = perm[t];
        perm[t] = pj;
        const uint32_t b = 1u << (pt & 31u);
#pragma unroll
        for (int w = 0; w < ChunkMask<S>::kWords; ++w) mask.w[w] |= ((pt >> 5) == w) ? b : 0u;
    }
    return mask;
}

// Compress half (top-k) on full tiles: chunks [0, 64*n_tiles), all complete.  Chunk sizes up
// to 64: beyond that a chunk no longer fits one lane at two wavefronts per SIMD, and the
// two-lanes-per-chunk kernels (pair_kernels.hip.h) take over.
template <int S, int K, bool GRAD_BF16, int VAL = 0>
__global__ __launch_bounds__(kWave, TileGeom<S>::kWavesPerSimd) void compress_tiled_topk(
    KParams p, int64_t n_tiles, TailRange tail, const void* __restrict__ grad,
    float* __restrict__ mom, void* __restrict__ idx_out, void* __restrict__ val_out,
    float* __restrict__ coeff_dbg) {
    using G = TileGeom<S>;
    constexpr int H = S / 2;
    __shared__ __attribute__((aligned(16))) char smem[G::kCompressBytes];
    float* tile = reinterpret_cast<float*>(smem);
    const int lane = threadIdx.x;
    // one tile per workgroup, then one tail chunk per surplus workgroup
    const int64_t t = blockIdx.x;
    if (t >= n_tiles) {
        compress_generic_chunks<GRAD_BF16>(p, tail.n, n_tiles * kWave + (t - n_tiles),
                                           tail.n_chunks, gridDim.x - n_tiles,
                                           *reinterpret_cast<GenericCompressSmem*>(smem), grad, mom,
                                           idx_out, val_out, coeff_dbg);
        return;
    }
    const int64_t ebase = t * G::kElems;

    fold_tile_to_lds<S, GRAD_BF16>(p, grad, mom, ebase, tile, lane);
    wave_lds_sync();

    // ---- phase 2: lane = chunk
    float* row = tile + lane * G::kRow;
    float c[S];
    row_to_regs<S>(row, c);
    FastDct<S>::dct2(c);
    c[0] *= p.alpha0;
    static_for<1, S>([&](auto i) { c[i] *= p.alpha; });
    if (coeff_dbg) regs_to_global<S>(coeff_dbg + ebase + static_cast<int64_t>(lane) * S, c);

    // threshold: K-th largest magnitude
    static_assert(S <= 64, "a chunk and its sorted magnitudes live in one lane's registers");
    uint32_t T;
    {
        uint32_t A[H], B[H];
        static_for<0, H>([&](auto i) {
            A[i] = __float_as_uint(c[i]) & 0x7FFFFFFFu;
            B[i] = __float_as_uint(c[H + i]) & 0x7FFFFFFFu;
        });
        sort_desc<H>(A);
        sort_desc<H>(B);
        T = kth_largest<H, K>(A, B);
    }
    // keep magnitude >= T: the mask collects the decisions (bit i = element i kept), and a
    // second register array u receives, in the same pass, what stays behind in the momentum
    // (the dropped coefficients)
    float u[S];
    ChunkMask<S> mk;
#pragma unroll
    for (int w = 0; w < ChunkMask<S>::kWords; ++w) mk.w[w] = 0u;
    static_for<0, S>([&](auto I) {
        constexpr int i = S - 1 - I;   // descending so that shifting lands bit i at i
        const bool keep = (__float_as_uint(c[i]) & 0x7FFFFFFFu) >= T;
        u[i] = keep ? 0.0f : c[i];
        mk.w[i / 32] = (mk.w[i / 32] << 1) | (keep ? 1u : 0u);
    });
    if (__any(mk.count() != K)) {
        // a tie at the threshold somewhere in this wavefront: exact rule, everything above
        // T plus the lowest-index entries equal to T
        int need = K;
        static_for<0, S>([&](auto i) {
            need -= ((__float_as_uint(c[i]) & 0x7FFFFFFFu) > T) ? 1 : 0;
        });
#pragma unroll
        for (int w = 0; w < ChunkMask<S>::kWords; ++w) mk.w[w] = 0u;
        static_for<0, S>([&](auto i) {
            const uint32_t key = __float_as_uint(c[i]) & 0x7FFFFFFFu;
            const bool take = (key == T) && (need > 0);
            need -= take ? 1 : 0;
            const bool keep = (key > T) || take;
            mk.w[i / 32] |= (keep ? 1u : 0u) << (i % 32);
            u[i] = keep ? 0.0f : c[i];
        });
    }

    if constexpr (VAL == 1 || VAL == 2) {
        // 16-bit transfer: the payload carries the rounded coefficient, and the rounding
        // error of a kept coefficient stays behind in the momentum with the dropped ones
        static_for<0, S>([&](auto i) {
            const float r = decode16<VAL>(encode16<VAL>(c[i]));
            u[i] = mk.bit(i) ? (c[i] - r) : c[i];
            c[i] = r;
        });
    }
    compact_and_store_payload<S, K, VAL>(c, mk, tile, lane, idx_out, val_out, t * (kWave * K));

    // ---- m <- m1 - q.  With q = D^T(kept coefficients) and m1 = D^T(all coefficients), the
    // residual is the inverse transform of the dropped ones.
    u[0] *= p.alpha0;
    static_for<1, S>([&](auto i) { u[i] *= p.alpha; });
    FastDct<S>::dct3(u);
    regs_to_row<S>(row, u);
    wave_lds_sync();
    store_tile_momentum<S>(tile, mom, ebase, lane);
}

// Compress half for Striding and Random on full tiles, in the raw-momentum domain or (with
// p.use_dct) on DCT coefficients.  Same three phases; the kept set is a bit pattern that does
// not depend on the data: `stride_mask` for Striding, a per-chunk shuffle for Random.
// VAL as in compact_and_store_payload (narrow formats: byte indices, if any are asked for).
template <int S, int K, bool GRAD_BF16, int VAL = 0>
__global__ __launch_bounds__(kWave, TileGeom<S>::kWavesPerSimd) void compress_tiled_scheme(
    KParams p, MaskWords stride_mask, int64_t n_tiles, TailRange tail,
    const void* __restrict__ grad, float* __restrict__ mom, void* __restrict__ idx_out,
    void* __restrict__ val_out, float* __restrict__ coeff_dbg) {
    using G = TileGeom<S>;
    __shared__ __attribute__((aligned(16))) char smem[G::kCompressBytes];
    float* tile = reinterpret_cast<float*>(smem);
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    if (t >= n_tiles) {
        compress_generic_chunks<GRAD_BF16>(p, tail.n, n_tiles * kWave + (t - n_tiles),
                                           tail.n_chunks, gridDim.x - n_tiles,
                                           *reinterpret_cast<GenericCompressSmem*>(smem), grad, mom,
                                           idx_out, val_out, coeff_dbg);
        return;
    }
    const int64_t ebase = t * G::kElems;

    fold_tile_to_lds<S, GRAD_BF16>(p, grad, mom, ebase, tile, lane);
    wave_lds_sync();

    float* row = tile + lane * G::kRow;
    float c[S];
    row_to_regs<S>(row, c);
    if (p.use_dct) {
        FastDct<S>::dct2(c);
        c[0] *= p.alpha0;
        static_for<1, S>([&](auto i) { c[i] *= p.alpha; });
    }
    if (coeff_dbg) regs_to_global<S>(coeff_dbg + ebase + static_cast<int64_t>(lane) * S, c);

    ChunkMask<S> mk = mask_from_words<S>(stride_mask);
    if (p.scheme == 2) {
        wave_lds_sync();   // rows are in registers: the tile doubles as shuffle scratch
        mk = random_mask<S, K>(p.seed, p.step, static_cast<uint64_t>(t) * kWave + lane,
                               reinterpret_cast<uint8_t*>(tile) + lane * G::kPermStride);
        wave_lds_sync();
    }

    if constexpr (VAL == 1 || VAL == 2) {
        // 16-bit transfer: the payload carries the rounded value; the rounding error of a
        // kept value stays behind in the momentum
        float u[S];
        static_for<0, S>([&](auto i) {
            const float r = decode16<VAL>(encode16<VAL>(c[i]));
            u[i] = mk.bit(i) ? (c[i] - r) : c[i];
            c[i] = r;
        });
        compact_and_store_payload<S, K, VAL>(c, mk, tile, lane, idx_out, val_out,
                                             t * (kWave * K));
        static_for<0, S>([&](auto i) { c[i] = u[i]; });
    } else {
        compact_and_store_payload<S, K, VAL>(c, mk, tile, lane, idx_out, val_out,
                                             t * (kWave * K));
        static_for<0, S>([&](auto i) { c[i] = mk.bit(i) ? 0.0f : c[i]; });
    }
    if (p.use_dct) {
        c[0] *= p.alpha0;
        static_for<1, S>([&](auto i) { c[i] *= p.alpha; });
        FastDct<S>::dct3(c);
    }
    regs_to_row<S>(row, c);
    wave_lds_sync();
    store_tile_momentum<S>(tile, mom, ebase, lane);
}

// One replica's payload entries of a tile, as each lane holds them after a coalesced load:
// K/4 vectors of four consecutive entries.  VAL = 0: int32 indices + fp32 values;
// VAL = 1/2: byte indices + bf16/fp16 values, kept packed (3 registers per four entries).
template <int K, int VAL>
struct PayloadRegs;

template <int K>
struct PayloadRegs<K, 0> {
    static constexpr int kVec = (K % 4 == 0) ? K / 4 : 1;
    int4 i[kVec];
    float4 v[kVec];
    __device__ __forceinline__ void load(int it, const void* ir, const void* vr, int e) {
        const uint4 iv = ld_u4<DETO_NT_DECOMPRESS_LD>(static_cast<const int32_t*>(ir) + e);
        i[it] = make_int4(iv.x, iv.y, iv.z, iv.w);
        v[it] = ld_f4<DETO_NT_DECOMPRESS_LD>(static_cast<const float*>(vr) + e);
    }
    template <int C>
    __device__ __forceinline__ uint32_t idx(int it) const {
        return static_cast<uint32_t>(C == 0 ? i[it].x : C == 1 ? i[it].y : C == 2 ? i[it].z : i[it].w);
    }
    template <int C>
    __device__ __forceinline__ float val(int it) const {
        return C == 0 ? v[it].x : C == 1 ? v[it].y : C == 2 ? v[it].z : v[it].w;
    }
};

template <int K, int VAL>
struct PayloadRegs {
    static constexpr int kVec = (K % 4 == 0) ? K / 4 : 1;
    uint32_t i[kVec];
    uint2 v[kVec];
    __device__ __forceinline__ void load(int it, const void* ir, const void* vr, int e) {
        i[it] = ld_u1<DETO_NT_DECOMPRESS_LD>(static_cast<const uint8_t*>(ir) + e);
        v[it] = ld_u2<DETO_NT_DECOMPRESS_LD>(static_cast<const uint16_t*>(vr) + e);
    }
    template <int C>
    __device__ __forceinline__ uint32_t idx(int it) const {
        return (i[it] >> (8 * C)) & 0xFFu;
    }
    template <int C>
    __device__ __forceinline__ float val(int it) const {
        const uint32_t w = (C < 2) ? v[it].x : v[it].y;
        return decode16<VAL>(static_cast<uint16_t>((C & 1) ? (w >> 16) : (w & 0xFFFFu)));
    }
};

// Ternary values + byte indices, K a multiple of 4: a chunk's two-bit codes start on a word
// boundary (ceil(K/16) words per chunk), and the four entries of a lane's vector are one byte.
template <int K>
struct PayloadRegs<K, 3> {
    static_assert(K % 4 == 0, "vector path");
    static constexpr int kVec = K / 4;
    static constexpr int kChunkBytes = 4 * ((K + 15) / 16);
    uint32_t i[kVec];
    uint32_t v[kVec];
    __device__ __forceinline__ void load(int it, const void* ir, const void* vr, int e) {
        i[it] = ld_u1<DETO_NT_DECOMPRESS_LD>(static_cast<const uint8_t*>(ir) + e);
        v[it] = static_cast<const uint8_t*>(vr)[(e / K) * kChunkBytes + (e % K) / 4];
    }
    template <int C>
    __device__ __forceinline__ uint32_t idx(int it) const {
        return (i[it] >> (8 * C)) & 0xFFu;
    }
    template <int C>
    __device__ __forceinline__ float val(int it) const {
        const uint32_t code = (v[it] >> (2 * C)) & 3u;
        return (code & 1u) ? ((code & 2u) ? -1.0f : 1.0f) : 0.0f;
    }
};

template <int K, int VAL>
__device__ __forceinline__ void load_payload(PayloadRegs<K, VAL>& r, const void* __restrict__ ir,
                                             const void* __restrict__ vr, int lane) {
    static_assert(K % 4 == 0, "vector path");
#pragma unroll
    for (int it = 0; it < K / 4; ++it) r.load(it, ir, vr, it * 256 + lane * 4);
}

// a[chunk][index] += value; an index outside [0,S) lands in the row's padding slot S.
// LDS floating-point atomics take several cycles per lane on this hardware, so the common
// case avoids them: when every chunk's indices are strictly ascending (what compress
// emits) all additions of one replica go to distinct accumulators and a plain
// read-all / add / write-all is exact.  Anything else (duplicates, disorder) takes the
// atomic path, which adds duplicates like the scatter-add it is.
template <int S, int K, int VAL>
__device__ __forceinline__ void scatter_payload(const PayloadRegs<K, VAL>& r, float* tile,
                                                int lane) {
    constexpr int kRow = S + 4;
    constexpr int kIt = K / 4;
    constexpr uint32_t kS = static_cast<uint32_t>(S);
    bool ok = true;
    [[maybe_unused]] uint32_t tail_prev = 0u;   // last index of lane 63's previous vector
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const uint32_t x = r.template idx<0>(it), y = r.template idx<1>(it),
                       z = r.template idx<2>(it), w = r.template idx<3>(it);
        // the lane's vector holds entries it*256 + 4*lane ... + 3: the first of its chunk?
        const bool first = ((it * 256 + lane * 4) % K) == 0;
        // previous lane's last index: a DPP shift inside the 16-lane row when chunks never
        // straddle rows (K/4 divides 16 and 256), a full-wavefront shift otherwise
        uint32_t pw;
        if constexpr (16 % kIt == 0)
            pw = static_cast<uint32_t>(
                __builtin_amdgcn_update_dpp(0, static_cast<int>(w), 0x111, 0xf, 0xf, false));
        else
            pw = static_cast<uint32_t>(__shfl_up(static_cast<int>(w), 1));
        // lane 0 may continue a chunk begun by lane 63 of the previous vector (only when K
        // does not divide 256; for it = 0 lane 0 is always the first of its chunk)
        if constexpr (256 % K != 0) {
            if (lane == 0) pw = tail_prev;
            tail_prev = static_cast<uint32_t>(
                __builtin_amdgcn_readlane(static_cast<int>(w), kWave - 1));
        }
        ok = ok && (x < y) && (y < z) && (z < w) && (first || pw < x);
    }
    if (!__any(!ok)) {
        // groups of a few vectors: all reads of a group, then all its writes
        constexpr int kGroup = kIt < 4 ? kIt : 4;
#pragma unroll
        for (int g0 = 0; g0 < kIt; g0 += kGroup) {
            float old[kGroup][4];
            float* at[kGroup][4];
#pragma unroll
            for (int g = 0; g < kGroup; ++g) {
                const int it = g0 + g;
                float* arow = tile + ((it * 256 + lane * 4) / K) * kRow;
                at[g][0] = arow + min(r.template idx<0>(it), kS);
                at[g][1] = arow + min(r.template idx<1>(it), kS);
                at[g][2] = arow + min(r.template idx<2>(it), kS);
                at[g][3] = arow + min(r.template idx<3>(it), kS);
#pragma unroll
                for (int c = 0; c < 4; ++c) old[g][c] = *at[g][c];
            }
#pragma unroll
            for (int g = 0; g < kGroup; ++g) {
                const int it = g0 + g;
                *at[g][0] = old[g][0] + r.template val<0>(it);
                *at[g][1] = old[g][1] + r.template val<1>(it);
                *at[g][2] = old[g][2] + r.template val<2>(it);
                *at[g][3] = old[g][3] + r.template val<3>(it);
            }
        }
    } else {
#pragma unroll
        for (int it = 0; it < kIt; ++it) {
            float* arow = tile + ((it * 256 + lane * 4) / K) * kRow;
            atomicAdd(arow + min(r.template idx<0>(it), kS), r.template val<0>(it));
            atomicAdd(arow + min(r.template idx<1>(it), kS), r.template val<1>(it));
            atomicAdd(arow + min(r.template idx<2>(it), kS), r.template val<2>(it));
            atomicAdd(arow + min(r.template idx<3>(it), kS), r.template val<3>(it));
        }
    }
}

// The tile's parameters, loaded early (needed only after the transform).
template <int S, bool PARAM_BF16>
struct ParamRegs {
    static constexpr int kIt = S / 8;
    uint4 b[PARAM_BF16 ? kIt : 1];
    float4 f[PARAM_BF16 ? 1 : 2 * kIt];
};

template <int S, bool PARAM_BF16>
__device__ __forceinline__ void load_params(ParamRegs<S, PARAM_BF16>& th,
                                            const void* __restrict__ params, int64_t ebase,
                                            int lane) {
#pragma unroll
    for (int it = 0; it < S / 8; ++it) {
        const int pe = it * 512 + lane * 8;
        if constexpr (PARAM_BF16) {
            th.b[it] =
                ld_u4<DETO_NT_DECOMPRESS_LD>(static_cast<const uint16_t*>(params) + ebase + pe);
        } else {
            const float* src = static_cast<const float*>(params) + ebase + pe;
            th.f[2 * it] = ld_f4<DETO_NT_DECOMPRESS_LD>(src);
            th.f[2 * it + 1] = ld_f4<DETO_NT_DECOMPRESS_LD>(src + 4);
        }
    }
}

// Last phase of decompress: the tile rows hold Q; theta <- theta*(1-eta*lambda) - eta*Q,
// coalesced, rounded to the parameter dtype.
template <int S, bool PARAM_BF16>
__device__ __forceinline__ void update_params_from_tile(const KParams& p, const float* tile,
                                                        const ParamRegs<S, PARAM_BF16>& th,
                                                        void* __restrict__ params, int64_t ebase,
                                                        int lane) {
    using G = TileGeom<S>;
#pragma unroll
    for (int it = 0; it < S / 8; ++it) {
        const int pe = it * 512 + lane * 8;
        const float* src = tile + (pe / S) * G::kRow + (pe % S);
        const float4 qa = *reinterpret_cast<const float4*>(src);
        const float4 qb = *reinterpret_cast<const float4*>(src + 4);
        if constexpr (PARAM_BF16) {
            uint16_t* dst = static_cast<uint16_t*>(params) + ebase + pe;
            const uint4 raw = th.b[it];
            auto upd = [&](uint32_t w, float q0, float q1) -> uint32_t {
                const float t0 = __uint_as_float(w << 16) * p.wd_scale;
                const float t1 = __uint_as_float(w & 0xFFFF0000u) * p.wd_scale;
                return pack_bf16x2(fmaf(-p.lr, q0, t0), fmaf(-p.lr, q1, t1));
            };
            uint4 out;
            out.x = upd(raw.x, qa.x, qa.y);
            out.y = upd(raw.y, qa.z, qa.w);
            out.z = upd(raw.z, qb.x, qb.y);
            out.w = upd(raw.w, qb.z, qb.w);
            st_u4<DETO_NT_DECOMPRESS_ST>(dst, out);
        } else {
            float* dst = static_cast<float*>(params) + ebase + pe;
            float4 ta = th.f[2 * it];
            float4 tb = th.f[2 * it + 1];
            ta.x = fmaf(-p.lr, qa.x, ta.x * p.wd_scale);
            ta.y = fmaf(-p.lr, qa.y, ta.y * p.wd_scale);
            ta.z = fmaf(-p.lr, qa.z, ta.z * p.wd_scale);
            ta.w = fmaf(-p.lr, qa.w, ta.w * p.wd_scale);
            tb.x = fmaf(-p.lr, qb.x, tb.x * p.wd_scale);
            tb.y = fmaf(-p.lr, qb.y, tb.y * p.wd_scale);
            tb.z = fmaf(-p.lr, qb.z, tb.z * p.wd_scale);
            tb.w = fmaf(-p.lr, qb.w, tb.w * p.wd_scale);
            st_f4<DETO_NT_DECOMPRESS_ST>(dst, ta);
            st_f4<DETO_NT_DECOMPRESS_ST>(dst + 4, tb);
        }
    }
}

// Last phase of decompress with Decoupled AdamW: the tile rows hold Q; the moments stream
// through (read, update, write) together with the parameters.  The moments of a batch of
// iterations are requested before the first is used: the stores of one iteration go to the
// arrays the next one loads from, so the compiler cannot move those loads up by itself.
template <int S, bool PARAM_BF16>
__device__ __forceinline__ void update_params_adamw_from_tile(const KParams& p, const float* tile,
                                                              const ParamRegs<S, PARAM_BF16>& th,
                                                              void* __restrict__ params,
                                                              const AdamPtrs& ad, int64_t ebase,
                                                              int lane) {
    using G = TileGeom<S>;
    constexpr int kIt = S / 8;
    constexpr int kBatch = kIt < 4 ? kIt : 4;
    static_assert(kIt % kBatch == 0, "whole batches");
    auto load8 = [&](const float* base, int pe, float (&x)[8]) {
        const float4 a = ld_f4<DETO_NT_DECOMPRESS_LD>(base + ebase + pe);
        const float4 b = ld_f4<DETO_NT_DECOMPRESS_LD>(base + ebase + pe + 4);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    };
    auto store8 = [&](float* base, int pe, const float (&x)[8]) {
        st_f4<DETO_NT_DECOMPRESS_ST>(base + ebase + pe, make_float4(x[0], x[1], x[2], x[3]));
        st_f4<DETO_NT_DECOMPRESS_ST>(base + ebase + pe + 4, make_float4(x[4], x[5], x[6], x[7]));
    };
#pragma unroll
    for (int b0 = 0; b0 < kIt; b0 += kBatch) {
        float m[kBatch][8], v[kBatch][8], vm[kBatch][8];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int pe = (b0 + j) * 512 + lane * 8;
            load8(ad.m, pe, m[j]);
            load8(ad.v, pe, v[j]);
            if (p.amsgrad) load8(ad.vmax, pe, vm[j]);
            else {
#pragma unroll
                for (int c = 0; c < 8; ++c) vm[j][c] = 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int it = b0 + j;
            const int pe = it * 512 + lane * 8;
            const float* src = tile + (pe / S) * G::kRow + (pe % S);
            const float4 qa = *reinterpret_cast<const float4*>(src);
            const float4 qb = *reinterpret_cast<const float4*>(src + 4);
            const float q[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
            float old[8], nw[8];
            if constexpr (PARAM_BF16) {
                const uint4 raw = th.b[it];
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    old[2 * c] = __uint_as_float(w[c] << 16);
                    old[2 * c + 1] = __uint_as_float(w[c] & 0xFFFF0000u);
                }
            } else {
                const float4 a = th.f[2 * it], b = th.f[2 * it + 1];
                old[0] = a.x; old[1] = a.y; old[2] = a.z; old[3] = a.w;
                old[4] = b.x; old[5] = b.y; old[6] = b.z; old[7] = b.w;
            }
#pragma unroll
            for (int c = 0; c < 8; ++c)
                nw[c] = adamw_step(p, old[c], q[c], m[j][c], v[j][c], vm[j][c]);
            store8(ad.m, pe, m[j]);
            store8(ad.v, pe, v[j]);
            if (p.amsgrad) store8(ad.vmax, pe, vm[j]);
            if constexpr (PARAM_BF16) {
                uint4 out;
                out.x = pack_bf16x2(nw[0], nw[1]);
                out.y = pack_bf16x2(nw[2], nw[3]);
                out.z = pack_bf16x2(nw[4], nw[5]);
                out.w = pack_bf16x2(nw[6], nw[7]);
                st_u4<DETO_NT_DECOMPRESS_ST>(static_cast<uint16_t*>(params) + ebase + pe, out);
            } else {
                store8(static_cast<float*>(params), pe, nw);
            }
        }
    }
}

// lane = chunk: scale the accumulated coefficients, inverse transform (if in the transform
// domain), optional export, sign, back into the lane's LDS row.
template <int S>
__device__ __forceinline__ void finish_chunk(const KParams& p, float (&y)[S], float* row,
                                             float* __restrict__ presign_dbg, int64_t ebase,
                                             int lane) {
    if (p.use_dct) {
        y[0] *= p.alpha0 * p.inv_R;
        const float ar = p.alpha * p.inv_R;
        static_for<1, S>([&](auto i) { y[i] *= ar; });
        FastDct<S>::dct3(y);
    } else {
        static_for<0, S>([&](auto i) { y[i] *= p.inv_R; });
    }
    if (presign_dbg) regs_to_global<S>(presign_dbg + ebase + static_cast<int64_t>(lane) * S, y);
    static_for<0, S>([&](auto i) { y[i] = sign_or_self(y[i], p.use_sign); });
    regs_to_row<S>(row, y);
}

// Four consecutive payload values as they are loaded (VAL = 0: fp32; 1 / 2: bf16 / fp16;
// 3: four two-bit signs in one byte), decoded only when they are used: a batch of loads can
// then be requested before the first wait.
template <int VAL>
struct RawQuad {
    uint2 w;
    __device__ __forceinline__ float4 get() const {
        return make_float4(decode16<VAL>(static_cast<uint16_t>(w.x & 0xFFFFu)),
                           decode16<VAL>(static_cast<uint16_t>(w.x >> 16)),
                           decode16<VAL>(static_cast<uint16_t>(w.y & 0xFFFFu)),
                           decode16<VAL>(static_cast<uint16_t>(w.y >> 16)));
    }
};
template <>
struct RawQuad<0> {
    float4 v;
    __device__ __forceinline__ float4 get() const { return v; }
};
template <>
struct RawQuad<3> {
    uint32_t b;
    __device__ __forceinline__ float4 get() const {
        auto dec = [](uint32_t code) { return (code & 1u) ? ((code & 2u) ? -1.0f : 1.0f) : 0.0f; };
        return make_float4(dec(b & 3u), dec((b >> 2) & 3u), dec((b >> 4) & 3u),
                           dec((b >> 6) & 3u));
    }
};

// One payload value as loaded, for the entry-by-entry paths (k < 4): fp32 bits, a 16-bit
// pattern, or (VAL = 3) the chunk's word of two-bit signs with the entry's number.
template <int VAL>
__device__ __forceinline__ float decode_entry(uint32_t raw, int j) {
    if constexpr (VAL == 0) {
        return __uint_as_float(raw);
    } else if constexpr (VAL == 3) {
        const uint32_t code = (raw >> (2 * j)) & 3u;
        return (code & 1u) ? ((code & 2u) ? -1.0f : 1.0f) : 0.0f;
    } else {
        return decode16<VAL>(static_cast<uint16_t>(raw));
    }
}

// Decompress-and-update half on full tiles, indices transmitted (top-k, or any scheme whose
// caller passes indices).  Several replicas' payloads (two to eight, by k) are in flight while
// one is scattered into LDS; LDS operations of one wavefront complete in order, so the additions
// into one accumulator happen replica after replica and the result does not depend on timing.
template <int S, int K, bool PARAM_BF16, int VAL = 0, bool ADAM = false>
__global__ __launch_bounds__(kWave, TileGeom<S>::kWavesPerSimd) void decompress_tiled(
    KParams p, int64_t n_tiles, TailRange tail, const void* __restrict__ idx_v,
    int64_t idx_stride, const void* __restrict__ val_v, int64_t val_stride,
    void* __restrict__ params, AdamPtrs ad, float* __restrict__ presign_dbg) {
    using G = TileGeom<S>;
    __shared__ __attribute__((aligned(16))) char smem[G::kDecompressBytes];
    float* tile = reinterpret_cast<float*>(smem);
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    if (t >= n_tiles) {
        decompress_generic_chunks<PARAM_BF16>(p, tail.n, n_tiles * kWave + (t - n_tiles),
                                              tail.n_chunks, gridDim.x - n_tiles,
                                              *reinterpret_cast<GenericDecompressSmem*>(smem),
                                              idx_v, idx_stride, val_v, val_stride, params, ad,
                                              presign_dbg);
        return;
    }
    const int64_t ebase = t * G::kElems;
    const int64_t pbase = t * (kWave * K);
    // replica r's entries of this tile, in bytes from the array bases
    // (ternary: ceil(K/16) words per chunk, replica stride in 32-bit words)
    constexpr int kIdxBytes = VAL ? 1 : 4, kValBytes = VAL ? 2 : 4;
    constexpr int kTernaryWords = (K + 15) / 16;
    const char* idx = static_cast<const char*>(idx_v) + pbase * kIdxBytes;
    const char* val = static_cast<const char*>(val_v) +
                      (VAL == 3 ? t * (kWave * kTernaryWords * 4) : pbase * kValBytes);
    const int64_t idx_step = idx_stride * kIdxBytes;
    const int64_t val_step = val_stride * (VAL == 3 ? 4 : kValBytes);

    // zero the accumulator tile
#pragma unroll
    for (int i = 0; i < G::kFloats / (kWave * 4); ++i)
        *reinterpret_cast<float4*>(tile + (i * kWave + lane) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_sync();
    if constexpr (K % 4 == 0) {
        // kBuf replicas' payloads in flight (as many as the registers allow: a replica's
        // entries are 2K registers in the widest format) while one is scattered; with a large
        // replication group and a small k every separate wait would cost a memory latency
        constexpr int kBuf = K > 32 ? 2 : (K > 8 ? 3 : 8);
        PayloadRegs<K, VAL> b[kBuf];
        auto fetch = [&](PayloadRegs<K, VAL>& dst, int r) {
            load_payload<K, VAL>(dst, idx + r * idx_step, val + r * val_step, lane);
        };
#pragma unroll
        for (int i = 0; i < kBuf; ++i)
            if (i < p.R) fetch(b[i], i);
        for (int r0 = 0; r0 < p.R; r0 += kBuf) {
#pragma unroll
            for (int i = 0; i < kBuf; ++i) {
                if (r0 + i < p.R) {
                    scatter_payload<S, K, VAL>(b[i], tile, lane);
                    if (r0 + i + kBuf < p.R) fetch(b[i], r0 + i + kBuf);
                }
            }
        }
    } else {
        // K entries per chunk, lane = chunk: the lane owns its row, plain sequential adds.
        // Eight replicas' entries are requested before the first is added.
        constexpr int kBatch = 8;
        float* arow = tile + lane * G::kRow;
        for (int r0 = 0; r0 < p.R; r0 += kBatch) {
            uint32_t at[kBatch][K];
            uint32_t raw[kBatch][K];    // values as loaded; VAL = 3: the chunk's word in raw[i][0]
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (r0 + i < p.R) {
                    const int r = r0 + i;
                    const char* ir = idx + r * idx_step + lane * K * kIdxBytes;
                    const char* vr = val + r * val_step;
                    if constexpr (VAL == 3) {
                        static_assert(K < 16, "one word per chunk");
                        raw[i][0] = reinterpret_cast<const uint32_t*>(vr)[lane];
                    }
#pragma unroll
                    for (int j = 0; j < K; ++j) {
                        if constexpr (VAL == 0) {
                            at[i][j] =
                                static_cast<uint32_t>(reinterpret_cast<const int32_t*>(ir)[j]);
                            raw[i][j] = reinterpret_cast<const uint32_t*>(vr)[lane * K + j];
                        } else {
                            at[i][j] = reinterpret_cast<const uint8_t*>(ir)[j];
                            if constexpr (VAL != 3)
                                raw[i][j] = reinterpret_cast<const uint16_t*>(vr)[lane * K + j];
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (r0 + i < p.R) {
#pragma unroll
                    for (int j = 0; j < K; ++j)
                        arow[min(at[i][j], static_cast<uint32_t>(S))] +=
                            decode_entry<VAL>(raw[i][VAL == 3 ? 0 : j], j);
                }
            }
        }
    }
    ParamRegs<S, PARAM_BF16> th;
    load_params<S, PARAM_BF16>(th, params, ebase, lane);
    wave_lds_sync();

    float* row = tile + lane * G::kRow;
    float y[S];
    row_to_regs<S>(row, y);
    finish_chunk<S>(p, y, row, presign_dbg, ebase, lane);
    wave_lds_sync();
    if constexpr (ADAM) update_params_adamw_from_tile<S, PARAM_BF16>(p, tile, th, params, ad, ebase, lane);
    else update_params_from_tile<S, PARAM_BF16>(p, tile, th, params, ebase, lane);
}

// Decompress-and-update half for Striding and Random without transmitted indices: every
// replica kept the same positions, so the R value arrays are summed entry by entry while
// they stream in, and each chunk's lane spreads the k sums over the positions of its bit
// pattern.
template <int S, int K, bool PARAM_BF16, bool ADAM = false, int VAL = 0>
__global__ __launch_bounds__(kWave, TileGeom<S>::kWavesPerSimd) void decompress_tiled_scheme(
    KParams p, MaskWords stride_mask, int64_t n_tiles, TailRange tail,
    const void* __restrict__ val_v, int64_t val_stride, void* __restrict__ params, AdamPtrs ad,
    float* __restrict__ presign_dbg) {
    using G = TileGeom<S>;
    __shared__ __attribute__((aligned(16))) char smem[G::kDecompressBytes];
    float* tile = reinterpret_cast<float*>(smem);
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    if (t >= n_tiles) {
        decompress_generic_chunks<PARAM_BF16>(p, tail.n, n_tiles * kWave + (t - n_tiles),
                                              tail.n_chunks, gridDim.x - n_tiles,
                                              *reinterpret_cast<GenericDecompressSmem*>(smem),
                                              nullptr, 0, val_v, val_stride, params, ad,
                                              presign_dbg);
        return;
    }
    const int64_t ebase = t * G::kElems;
    const int64_t pbase = t * (kWave * K);
    constexpr int PR = staging_row(K);
    static_assert(kWave * PR * 4 + kWave * G::kPermStride <= G::kFloats * 4, "LDS layout");

    ParamRegs<S, PARAM_BF16> th;
    load_params<S, PARAM_BF16>(th, params, ebase, lane);

    // sum over replicas, coalesced; staged as [chunk][k].  One replica's four consecutive
    // entries it*256 + 4*lane ... of this tile, as loaded (k a multiple of 4):
    [[maybe_unused]] auto load4 = [&](int r, int it) -> RawQuad<VAL> {
        const int e = it * 256 + lane * 4;
        RawQuad<VAL> q;
        if constexpr (VAL == 0) {
            q.v = ld_f4<DETO_NT_DECOMPRESS_LD>(static_cast<const float*>(val_v) + r * val_stride +
                                               pbase + e);
        } else if constexpr (VAL == 3) {
            // two-bit signs: ceil(K/16) words per chunk, replica stride in words
            constexpr int kChunkBytes = 4 * ((K + 15) / 16);
            const uint8_t* bytes = static_cast<const uint8_t*>(val_v) + r * val_stride * 4 +
                                   t * (kWave * kChunkBytes);
            q.b = bytes[(e / K) * kChunkBytes + (e % K) / 4];
        } else {
            q.w = ld_u2<DETO_NT_DECOMPRESS_LD>(static_cast<const uint16_t*>(val_v) +
                                               r * val_stride + pbase + e);
        }
        return q;
    };
    if constexpr (K % 4 == 0) {
        float4 acc[K / 4];
#pragma unroll
        for (int it = 0; it < K / 4; ++it) acc[it] = load4(0, it).get();
        // the other replicas in batches: all loads of a batch are requested before the first
        // is added (a large replication group with a small k would otherwise pay a memory
        // latency per replica); the order of the additions stays r = 0, 1, 2, ...
        constexpr int kBatch = K >= 32 ? 2 : (K >= 16 ? 4 : 8);
        for (int r0 = 1; r0 < p.R; r0 += kBatch) {
            RawQuad<VAL> nxt[kBatch][K / 4];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (r0 + i < p.R) {
#pragma unroll
                    for (int it = 0; it < K / 4; ++it) nxt[i][it] = load4(r0 + i, it);
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (r0 + i < p.R) {
#pragma unroll
                    for (int it = 0; it < K / 4; ++it) {
                        const float4 v = nxt[i][it].get();
                        acc[it].x += v.x; acc[it].y += v.y;
                        acc[it].z += v.z; acc[it].w += v.w;
                    }
                }
            }
        }
#pragma unroll
        for (int it = 0; it < K / 4; ++it) {
            const int e = it * 256 + lane * 4;
            *reinterpret_cast<float4*>(tile + (e / K) * PR + (e % K)) = acc[it];
        }
    } else {
        // k = 1, 2 (3): the lane sums its own chunk's entries, eight replicas per batch of loads
        constexpr int kBatch = 8;
        float a[K];
#pragma unroll
        for (int j = 0; j < K; ++j) a[j] = 0.0f;
        for (int r0 = 0; r0 < p.R; r0 += kBatch) {
            uint32_t x[kBatch][K];      // as loaded; VAL = 3: the chunk's word in x[i][0]
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (r0 + i < p.R) {
                    const int64_t r = r0 + i;
                    if constexpr (VAL == 3) {
                        static_assert(K < 16, "one word per chunk");
                        x[i][0] =
                            static_cast<const uint32_t*>(val_v)[r * val_stride + t * kWave + lane];
                    } else if constexpr (VAL == 0) {
#pragma unroll
                        for (int j = 0; j < K; ++j)
                            x[i][j] = static_cast<const uint32_t*>(
                                val_v)[r * val_stride + pbase + lane * K + j];
                    } else {
#pragma unroll
                        for (int j = 0; j < K; ++j)
                            x[i][j] = static_cast<const uint16_t*>(
                                val_v)[r * val_stride + pbase + lane * K + j];
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (r0 + i < p.R) {
#pragma unroll
                    for (int j = 0; j < K; ++j)
                        a[j] += decode_entry<VAL>(x[i][VAL == 3 ? 0 : j], j);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < K; ++j) tile[lane * PR + j] = a[j];
    }
    ChunkMask<S> mk = mask_from_words<S>(stride_mask);
    if (p.scheme == 2)
        mk = random_mask<S, K>(p.seed, p.step, static_cast<uint64_t>(t) * kWave + lane,
                               reinterpret_cast<uint8_t*>(tile + kWave * PR) +
                                   lane * G::kPermStride);
    wave_lds_sync();

    // lane = chunk: y[i] = kept ? sum[rank of i among the kept] : 0
    float y[S];
    {
        const float* vrow = tile + lane * PR;
        int pos = 0;
        static_for<0, S>([&](auto i) {
            const uint32_t bit = mk.bit(i);
            const float v = vrow[pos];
            y[i] = bit ? v : 0.0f;
            pos += static_cast<int>(bit);
        });
    }
    wave_lds_sync();
    float* row = tile + lane * G::kRow;
    finish_chunk<S>(p, y, row, presign_dbg, ebase, lane);
    wave_lds_sync();
    if constexpr (ADAM) update_params_adamw_from_tile<S, PARAM_BF16>(p, tile, th, params, ad, ebase, lane);
    else update_params_from_tile<S, PARAM_BF16>(p, tile, th, params, ebase, lane);
}

}  // namespace deto
