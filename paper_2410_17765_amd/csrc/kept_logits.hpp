// Logits kept by the forward pass for the backward pass (CP_HEAD_KEEP_LOGITS), matrix-core path.
//
// The forward product's epilogue writes zs[m, v] = fp16(z[m, v] - ref[m, v / 128]) with ref the maximum of row m
// over its block of 128 columns, which is also the first half of the (max, sum of exponentials) pair of that
// block in part[m, parts].  With the row's log-normaliser lse[m] the log-probability of eq. 5 is
//     log P[m, v] = zs[m, v] - (lse[m] - ref[m, v / 128]).
// Relative to the block maximum the large probabilities of a row sit near zero, where fp16 resolves 2^-12 or
// better; an overflow to -inf is the exact zero that the exponential of the true value rounds to as well.
//
// k_dz_from_kept turns a chunk of kept logits into logit gradients in bf16, row-major and (optionally)
// transposed, which is what the dY and dU products of the backward pass read (the row-major copy optionally block by
// block, the layout the dY product streams best).  What the gradient is (training
// loss, fine-tuning loss) comes in as a rule.
#pragma once
#include "gemm_nt.hpp"

namespace cph {

constexpr int kKeptTile = 128;      // rows and columns of a workgroup's tile; its columns are one block of `part`
constexpr int kKeptBlock = 256;

// 16-bit float (IEEE binary16) bit patterns, round to nearest even
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

struct KeptLogits {
    const uint16_t *zs;      // [rows, ld] fp16 bits
    const float2 *part;      // [rows, parts] {block maximum, -}
    long ld;
    int parts;
};

// log P for 8 consecutive columns col .. col + 7 (one block of 128) of row m, given the row's log-normaliser
__device__ __forceinline__ void kept_log_probs(const KeptLogits &k, size_t m, int col, float lse, float (&lp)[8])
{
    const float off = lse - k.part[m * k.parts + col / kKeptTile].x;
    const f16x8_t z = __builtin_bit_cast(f16x8_t, *reinterpret_cast<const u32x4_t *>(k.zs + m * k.ld + col));
#pragma unroll
    for (int j = 0; j < 8; ++j) lp[j] = (float)z[j] - off;
}

// A workgroup takes 128 rows x 128 columns of the chunk.  A thread owns Rule::RT consecutive rows (2, 4 or 8) and
// 8 consecutive columns: it reads their kept logits with 16-byte loads, lets the rule turn the log-probabilities
// into gradients, writes them row-major with 16-byte stores and leaves them, one 32-bit word per column and pair
// of rows, in a column-major LDS tile from which the transposed copy goes out in 16-byte pieces of 256-byte
// column segments.  The 16-byte pieces of an LDS column are stored at position (piece ^ column / 8): the
// sixteen threads that write the same rows address columns 8 apart, a multiple of the bank cycle otherwise.
//
// Rule: static constexpr int RT; and
//   void operator()(int row, int nrows, int col, int V, const float4 (&info)[RT], const float (&lp)[RT][8],
//                   float (&g)[RT][8]) const
// with row chunk-relative, rows row .. row + nrows - 1 valid (info = rowinfo of those rows, info.x their
// log-normaliser), g preset to zero; entries of columns >= V must stay zero.
// kept: rows of the chunk (already offset); rowinfo chunk-relative.  dZt may be null.
template <class Rule>
__global__ void __launch_bounds__(kKeptBlock) k_dz_from_kept(KeptLogits kept, const float4 *__restrict__ rowinfo,
                                                             Rule rule, int Mc, int Mcp, int V, int Vp,
                                                             bf16_t *__restrict__ dZ, long ldz, int dz_blocked,
                                                             bf16_t *__restrict__ dZt, long ldzt, int tiles_c)
{
    constexpr int RT = Rule::RT;
    static_assert(RT == 2 || RT == 4 || RT == 8, "pairs of rows are packed for the transposed copy");
    constexpr int CS = kKeptTile * 2 + 16;              // padded column stride in bytes
    __shared__ __align__(16) char stage[kKeptTile * CS];
    const int tc = blockIdx.x % tiles_c, tr = blockIdx.x / tiles_c;
    const int t = threadIdx.x, cg = t & 15;
    const int col = tc * kKeptTile + cg * 8;
    const bool col_in = col < Vp;                        // Vp is a multiple of 8: all eight columns or none
#pragma unroll
    for (int pass = 0; pass < kKeptTile / (16 * RT); ++pass) {
        const int rg = pass * 16 + (t >> 4);             // group of RT rows inside the tile
        const int row = tr * kKeptTile + RT * rg;
        float g[RT][8];
#pragma unroll
        for (int h = 0; h < RT; ++h)
#pragma unroll
            for (int k = 0; k < 8; ++k) g[h][k] = 0.f;
        if (col_in && row < Mc) {
            const int nrows = Mc - row < RT ? Mc - row : RT;
            float4 info[RT];
            float lp[RT][8];
#pragma unroll
            for (int h = 0; h < RT; ++h) {
                info[h] = rowinfo[row + (h < nrows ? h : 0)];
                kept_log_probs(kept, (size_t)(row + (h < nrows ? h : 0)), col, info[h].x, lp[h]);
            }
            rule(row, nrows, col, V, info, lp, g);
#pragma unroll
            for (int h = 0; h < RT; ++h)
                if (h < nrows) {
                    u32x4_t out;
#pragma unroll
                    for (int k = 0; k < 4; ++k) out[k] = f32x2_to_bf16x2(g[h][2 * k], g[h][2 * k + 1]);
                    const size_t at = dz_blocked ? blocked64_index((size_t)(row + h), col, ldz) : (size_t)(row + h) * ldz + col;
                    *reinterpret_cast<u32x4_t *>(dZ + at) = out;
                }
        }
        if (dZt) {
#pragma unroll
            for (int hp = 0; hp < RT / 2; ++hp) {
                const int rp = (RT / 2) * rg + hp;       // pair of rows inside the tile
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    *reinterpret_cast<uint32_t *>(stage + (cg * 8 + k) * CS + 16 * ((rp >> 2) ^ cg) + 4 * (rp & 3)) =
                        f32x2_to_bf16x2(g[2 * hp][k], g[2 * hp + 1][k]);
            }
        }
    }
    if (!dZt) return;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kKeptTile * 16 / kKeptBlock; ++q) {
        const int idx = q * kKeptBlock + t;
        const int c = idx >> 4, pos = idx & 15;
        const int piece = pos ^ (c >> 3);                // rows 8 piece .. 8 piece + 7 of the tile
        const u32x4_t val = *reinterpret_cast<const u32x4_t *>(stage + c * CS + pos * 16);
        const int grow = tr * kKeptTile + piece * 8, gcol = tc * kKeptTile + c;
        if (grow < Mcp && gcol < V) *reinterpret_cast<u32x4_t *>(dZt + (size_t)gcol * ldzt + grow) = val;
    }
}

// kept: all rows (not offset); the chunk is rows m0 .. m0 + Mc - 1; rowinfo chunk-relative.  ldz = Vp.
// dz_blocked: dZ is written block by block (blocked64_index) instead of row-major.
template <class Rule>
inline void launch_dz_from_kept(const KeptLogits &kept, size_t m0, const float4 *rowinfo, const Rule &rule, int Mc, int Mcp,
                                int V, bf16_t *dZ, long ldz, bool dz_blocked, bf16_t *dZt, long ldzt, hipStream_t st)
{
    const int Vp = (int)ldz;
    const int tiles_c = (Vp + kKeptTile - 1) / kKeptTile;
    const size_t tiles_r = ((size_t)Mcp + kKeptTile - 1) / kKeptTile;
    // algorithmic traffic: the logits read once, the gradients written once or twice
    ProfileScope scope("dz_from_kept", (double)Mc * Vp * 2.0 * (dZt ? 3.0 : 2.0), st);
    const KeptLogits chunk{kept.zs + m0 * kept.ld, kept.part + m0 * kept.parts, kept.ld, kept.parts};
    k_dz_from_kept<Rule><<<(unsigned)(tiles_r * tiles_c), kKeptBlock, 0, st>>>(chunk, rowinfo, rule, Mc, Mcp, V, Vp, dZ, ldz,
                                                                               dz_blocked ? 1 : 0, dZt, ldzt, tiles_c);
}

}  // namespace cph
