// Packed-delta layout shared by the pack/unpack kernels and the streaming kernels.
//
// What is stored (paper Section 4.1 steps 2-3): per group of four consecutive k the two kept
// values as b-bit codes plus their 2-bit positions, and one fp16 (scale, zero) per row and
// quantisation group.  How it is ordered is chosen for gfx950: the unit is a *tile* of 16 rows x
// 256 dense columns, cut into four *steps* of 64 columns, each step being exactly one
// V_SMFMAC_F32_16X16X64_F16 A-operand (A = sparse 16x64 held as 16x32 kept values + 2-bit
// positions).  In that instruction lane l = 16*q + r (r = row 0..15, q = 0..3) holds the eight
// kept values of dense columns 16q .. 16q+15 of row r -- four groups of four, two kept values
// each -- and a 16-bit field of position codes, kept slot e at bits [2e+1:2e].  A tile stores,
// lane by lane, exactly what that lane feeds to the four steps, so a wave streams a tile with one
// 16-byte (codes) and at most one 8-byte (positions) load per lane, fully coalesced.
//
//   tile index      ti = (n/16) * (K/256) + k/256
//   4-bit:  plane C  at byte 0                : ti*1024 + 16*l : uint4, dword s = codes of step s
//           plane I  at byte (N/16)(K/256)*1024: ti*512 + 8*l  : uint2, dword h = positions of
//                                                 steps 2h (low 16 bits) and 2h+1 (high 16 bits)
//           code of kept slot e (pair j = e/2, half h = e%2) sits at bit 16h + 4j of its dword
//   2-bit:  plane C  at byte 0                : ti*1024 + 16*l : uint4 {c01, c23, i01, i23}
//           c01 = codes of steps 0 (bits 0-7 / 16-23) and 1 (bits 8-15 / 24-31):
//           code of slot e of step s sits at bit 16h + 8(s%2) + 2j; i01/i23 as plane I above
//   scales: plane S after the planes above     : ti*(16*GPT*4) + (r*GPT + g)*4 : {scale, zero}
//           fp16 pair, GPT = 256/G quantisation groups per tile row
//
// With "pair j at bit 4j (or 2j) of both halves", (w >> shift) & 0x000F000F lands two codes in the
// two mantissas of a packed fp16 pair at once.
#pragma once
#include <stdint.h>
#include <stddef.h>

#ifndef DZ_HD
#ifdef __HIPCC__
#define DZ_HD __host__ __device__ inline
#else
#define DZ_HD inline
#endif
#endif

struct DzLayout {
    int N, K, bits, group;
    int RT, KT, GPT;            // row tiles, k tiles, quantisation groups per tile row
    size_t off_idx;             // byte offset of plane I (4-bit only)
    size_t off_scale;           // byte offset of plane S
    size_t total;
};

DZ_HD DzLayout dz_make_layout(int N, int K, int bits, int group)
{
    DzLayout L;
    L.N = N; L.K = K; L.bits = bits; L.group = group;
    L.RT = N / 16; L.KT = K / 256; L.GPT = 256 / group;
    size_t tiles = (size_t)L.RT * L.KT;
    if (bits == 4) { L.off_idx = tiles * 1024; L.off_scale = tiles * 1536; }
    else           { L.off_idx = 0;            L.off_scale = tiles * 1024; }
    L.total = L.off_scale + tiles * 16 * (size_t)L.GPT * 4;
    return L;
}

// The quantisation-only format (no 2:4 pruning: a b-bit code for every column; Section 4.1 step 3
// alone).  A dense group of four columns is the sum of two 2:4 patterns with fixed positions, columns
// {0, 1} (half 0) and columns {2, 3} (half 1); each half of a tile is stored exactly like plane C of
// a 2:4 tile whose kept columns are those two, so the sparse MFMA multiplies it with a constant
// position word and no positions are stored:
//   4-bit:  tile at ti*2048: half h at +1024h + 16*l : uint4, dword s = codes of step s
//   2-bit:  tile at ti*1024 + 16*l : uint4 {half 0: c01, c23, half 1: c01, c23}
//   scales: plane S as above, after all tiles
DZ_HD DzLayout dz_make_qlayout(int N, int K, int bits, int group)
{
    DzLayout L;
    L.N = N; L.K = K; L.bits = bits; L.group = group;
    L.RT = N / 16; L.KT = K / 256; L.GPT = 256 / group;
    size_t tiles = (size_t)L.RT * L.KT;
    L.off_idx = 0;
    L.off_scale = tiles * (bits == 4 ? 2048 : 1024);
    L.total = L.off_scale + tiles * 16 * (size_t)L.GPT * 4;
    return L;
}

// dword index and bit shift of the code of (row n, column k) in a quantisation-only blob
DZ_HD size_t dz_qcode_dword(const DzLayout &L, int n, int k)
{
    int kt = k >> 8, kin = k & 255;
    int s = kin >> 6, q = (kin & 63) >> 4, h = (kin & 3) >> 1;
    size_t tile = (size_t)(n >> 4) * L.KT + kt;
    int lane = q * 16 + (n & 15);
    if (L.bits == 4) return (tile * 2048 + (size_t)h * 1024 + (size_t)lane * 16) / 4 + s;
    return (tile * 1024 + (size_t)lane * 16) / 4 + 2 * h + (s >> 1);
}
DZ_HD int dz_qcode_shift(const DzLayout &L, int k)
{
    int kin = k & 255;
    int s = kin >> 6, j = (kin & 15) >> 2, hh = kin & 1;
    if (L.bits == 4) return 16 * hh + 4 * j;
    return 16 * hh + 8 * (s & 1) + 2 * j;
}

// Where kept entry (row n, kept column kk in [0, K/2)) lives.
struct DzSlot {
    size_t tile; int lane; int step; int e;     // e = kept slot 0..7 inside the lane's step
};

DZ_HD DzSlot dz_slot_of(const DzLayout &L, int n, int kk)
{
    DzSlot s;
    int k4 = kk >> 1;                 // group of four along k
    int k = k4 * 4;                   // its first dense column
    int kt = k >> 8, kin = k & 255;
    s.tile = (size_t)(n >> 4) * L.KT + kt;
    s.step = kin >> 6;
    int q = (kin & 63) >> 4;
    int j = (kin & 15) >> 2;
    s.lane = q * 16 + (n & 15);
    s.e = 2 * j + (kk & 1);
    return s;
}

DZ_HD size_t dz_code_dword(const DzLayout &L, const DzSlot &s)      // dword index into the blob
{
    if (L.bits == 4) return (s.tile * 1024 + (size_t)s.lane * 16) / 4 + s.step;
    return (s.tile * 1024 + (size_t)s.lane * 16) / 4 + (s.step >> 1);
}
DZ_HD int dz_code_shift(const DzLayout &L, const DzSlot &s)
{
    int j = s.e >> 1, h = s.e & 1;
    if (L.bits == 4) return 16 * h + 4 * j;
    return 16 * h + 8 * (s.step & 1) + 2 * j;
}
DZ_HD size_t dz_idx_dword(const DzLayout &L, const DzSlot &s)
{
    if (L.bits == 4) return (L.off_idx + s.tile * 512 + (size_t)s.lane * 8) / 4 + (s.step >> 1);
    return (s.tile * 1024 + (size_t)s.lane * 16) / 4 + 2 + (s.step >> 1);
}
DZ_HD int dz_idx_shift(const DzSlot &s) { return 16 * (s.step & 1) + 2 * s.e; }

// dword index of the {scale, zero} pair of (row n, quantisation group gq = k / G)
DZ_HD size_t dz_scale_dword(const DzLayout &L, int n, int gq)
{
    int kt = gq / L.GPT, g = gq % L.GPT;
    size_t tile = (size_t)(n >> 4) * L.KT + kt;
    return L.off_scale / 4 + tile * 16 * L.GPT + (size_t)(n & 15) * L.GPT + g;
}
