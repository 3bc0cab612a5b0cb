// Where the operand slabs of the matmul kernels sit in LDS: which global cell every lane of a direct load
// fetches, and where every lane reads its MFMA operand fragments.  Pure index arithmetic, usable on the host
// (the layout tests emulate a whole slab with these very functions) and in the kernels.
//
// A direct load (global_load_lds_dwordx4) moves 64 cells of 16 bytes: lane l fetches a cell of its own choice
// and it lands at the chunk's LDS address + 16 l.  Rows can therefore not be padded against bank conflicts;
// cells are swizzled instead, by the choice of each lane's source cell.
#pragma once

#if defined(__HIPCC__)
#define DASH_HD __host__ __device__ __forceinline__
#else
#define DASH_HD inline
#endif

namespace dash {
namespace layout {

// ---- 16-bit operands: slabs of TILE rows x HBK k, NW wavefronts --------------------------------------------
//   KC  element (row, k) at global base[row*ld + k] (k contiguous): LDS rows of HBK elements, cell q (eight k)
//       of row r at cell q ^ kc_swizzle(r); an MFMA operand (eight consecutive k of one row) is one 16-byte read.
//       Sixteen consecutive rows at one q - what sixteen lanes of such a read touch - fall into sixteen
//       different 16-byte bank groups.
//   KR  element (row, k) at global base[k*ld + row] (row contiguous): LDS k-lines of TILE elements, cell c
//       (eight rows) of line k at cell c ^ kr_swizzle(k); an MFMA operand is two transposing reads
//       (ds_read_b64_tr_b16): sixteen lanes j address line kk + j/4, rows rs + 4 (j%4) .. +3 and lane j receives
//       row rs + j of the four lines kk .. kk+3.  The four lines x four cells thirty-two lanes touch fall into
//       sixteen different bank groups.
template <int TILE, int HBK, int NW>
struct Half {
    static constexpr int HKQ = HBK / 8;                 // 16-byte cells per row of a KC slab
    static constexpr int RPC = 64 / HKQ;                // rows of a KC slab per chunk
    static constexpr int CHUNKS = TILE * HBK / 512;     // chunks of 1 KB per operand slab
    static constexpr int NV = CHUNKS / NW;              // loads per wavefront, operand and slab
    static constexpr int CPR = TILE / 8;                // 16-byte cells per k-line of a KR slab
    static constexpr int LPC = 64 / CPR;                // k-lines of a KR slab per chunk
    static constexpr int SLAB = TILE * HBK * 2;         // bytes of one operand slab
    static constexpr int STEPS = HBK / 16;              // MFMA steps (16 k) per slab
    static_assert(CHUNKS % NW == 0 && NV >= 1, "chunks must divide over the wavefronts");

    static DASH_HD int kc_swizzle(int row) { return HKQ == 8 ? (row >> 1) & 7 : (row >> 2) & 3; }
    static DASH_HD int kr_swizzle(int k) { return CPR >= 16 ? 4 * (k & 3) : 4 * ((k >> 1) & 1); }

    // chunk that load u of a wavefront fills: LDS bytes [1024 chunk, 1024 chunk + 1024) of the operand slab
    static DASH_HD int chunk(int wave, int u) { return wave + NW * u; }

    // byte offset, inside the block and without the part that moves with the slab, of the cell a lane fetches
    // in load u (32 bits suffice: a block has at most 16384^2 * 2 bytes).  row0 = first row of the tile.
    static DASH_HD unsigned load_offset(bool kc, int ld, int row0, int wave, int lane, int u) {
        const int ch = chunk(wave, u);
        if (kc) {
            const int row = RPC * ch + lane / HKQ;
            const int q = (lane % HKQ) ^ kc_swizzle(row);
            return ((unsigned)(row0 + row) * (unsigned)ld + 8u * q) * 2u;
        }
        const int k = LPC * ch + lane / CPR;
        const int c = (lane % CPR) ^ kr_swizzle(k);
        return ((unsigned)k * (unsigned)ld + row0 + 8u * c) * 2u;
    }

    // Fragment of MFMA step st for the 32-row sub-tile i of a wavefront whose sub-tiles start at r0: lane L holds
    // row r0 + 32 i + L%32, k = 16 st + 8 (L/32) + 0..7.
    // KC: byte offset of the 16-byte read = frag_kc(r0, lane, st) + i * KC_SUB
    static constexpr int KC_SUB = 32 * HBK * 2;
    static DASH_HD int frag_kc(int r0, int lane, int st) {
        const int row = r0 + (lane & 31);
        return row * (HBK * 2) + (((2 * st + (lane >> 5)) ^ kc_swizzle(row)) << 4);
    }
    // KR: byte offsets of the two transposing 8-byte reads = frag_kr(r0, i, lane) + st * KR_STEP (+ KR_HALF)
    static constexpr int KR_STEP = 16 * CPR * 16;
    static constexpr int KR_HALF = 4 * CPR * 16;
    static DASH_HD int frag_kr(int r0, int i, int lane) {
        const int j = lane & 15;
        const int kk = 8 * (lane >> 5) + (j >> 2);
        const int rs = r0 + 32 * i + 16 * ((lane >> 4) & 1) + 4 * (j & 3);
        return (kk * CPR + ((rs >> 3) ^ kr_swizzle(kk))) * 16 + 8 * (j & 1);
    }
};

// ---- fp32 operands: slabs of TILE rows x BK k, NW wavefronts; offsets in floats ------------------------------
//   KC  rows of BK floats, cell q (four k) of row r at q ^ kc_swizzle(r): one 16-byte read gives a lane its
//       operand for four consecutive MFMAs (k = 8c + 4 (lane/32) + s, s = 0..3).
//   RC  k-lines of TILE floats, float r of line k at r ^ rc_swizzle(k): four 4-byte reads, one per MFMA; the two
//       lines k and k + 4 that the lane halves touch fall into different halves of the 64 banks.
template <int TILE, int BK, int NW>
struct F32 {
    static constexpr int KQ = BK / 4;                   // 16-byte cells per row of a KC slab
    static constexpr int SLAB = TILE * BK;              // floats per operand slab
    static constexpr int CHUNKS = TILE * BK / 256;
    static constexpr int NV = CHUNKS / NW;
    static constexpr int RPC = 64 / KQ;
    static constexpr int CPR = TILE / 4;
    static constexpr int LPC = 64 / CPR;
    static_assert(CHUNKS % NW == 0 && NV >= 1, "chunks must divide over the wavefronts");

    static DASH_HD int kc_swizzle(int row) { return KQ == 8 ? (row >> 1) & 7 : (row >> 2) & 3; }
    static DASH_HD int rc_swizzle(int k) { return 32 * ((k >> 2) & 1); }
    static DASH_HD int chunk(int wave, int u) { return wave + NW * u; }

    static DASH_HD unsigned load_offset(bool kc, int ld, int row0, int wave, int lane, int u) {
        const int ch = chunk(wave, u);
        if (kc) {
            const int row = RPC * ch + lane / KQ;
            const int q = (lane % KQ) ^ kc_swizzle(row);
            return ((unsigned)(row0 + row) * (unsigned)ld + 4u * q) * 4u;
        }
        const int k = LPC * ch + lane / CPR;
        const int r = (4 * (lane % CPR)) ^ rc_swizzle(k);
        return ((unsigned)k * (unsigned)ld + row0 + r) * 4u;
    }

    // chunk c of 8 k, 32-row sub-tile i: lane L holds row r0 + 32 i + L%32 and k = 8c + 4 (L/32) + s, s = 0..3
    // KC: float offset of the 16-byte read = frag_kc(r0, lane, c) + i * KC_SUB
    static constexpr int KC_SUB = 32 * BK;
    static DASH_HD int frag_kc(int r0, int lane, int c) {
        const int rr = r0 + (lane & 31);
        return rr * BK + 4 * ((2 * c + (lane >> 5)) ^ kc_swizzle(rr));
    }
    // RC: float offset of the 4-byte read of step s = frag_rc(r0, i, lane) + (8 c + s) * TILE
    // (bit 2 of k = 8c + 4 (lane/32) + s is lane/32, whatever c and s)
    static DASH_HD int frag_rc(int r0, int i, int lane) {
        return 4 * (lane >> 5) * TILE + ((r0 + 32 * i + (lane & 31)) ^ (32 * (lane >> 5)));
    }
};

}  // namespace layout
}  // namespace dash
