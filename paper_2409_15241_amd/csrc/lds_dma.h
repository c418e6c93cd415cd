// Direct-to-LDS operand tiles for the GEMM: buffer_load ... lds writes global data straight into LDS
// (no VGPR staging, no ds_write), several tiles deep, and MFMA fragments are read back with
// ds_read_b128 (contraction-contiguous operands) or ds_read_b64_tr_b16 (contraction-strided operands:
// the transposing read of gfx950 delivers 4 consecutive contraction values per lane from a
// row-major [k][n] tile).
//
// A tile holds DMA_BK = 32 contraction elements.  One buffer_load_dwordx4 ... lds of a wave fills
// 1 KiB of LDS linearly (lane l writes bytes [16 l, 16 l + 16) from the LDS base in M0), so the
// swizzles below are applied on the GLOBAL side: each lane fetches the chunk that belongs at its
// fixed LDS position.  Lanes whose chunk lies outside the operand read at BUF_OOB and store zeros.
//
//   KC tile [R rows][32 k]   : chunk (r, kc) of 8 k at 16-byte slot  4 r + (kc ^ ((r >> 2) & 3)).
//       A fragment read (16 consecutive rows, one chunk index) touches 16 distinct bank groups.
//   KS tile [32 k][R rows]   : element (k, n) at byte  2 R k + 64 ((n >> 5) ^ (k & 3)) + 2 (n & 31).
//       A transposing read covers 4 consecutive k rows x 16 n: the XOR puts the 4 rows in 4
//       different 64-byte bank quarters.
#pragma once
#include "common.h"

typedef __amdgpu_buffer_rsrc_t buf_rsrc;
constexpr uint32_t BUF_OOB = 0x80000000u;      // operands are validated to be smaller than 2 GiB
constexpr int DMA_BK = 32;
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

DEV buf_rsrc make_rsrc(const void* base, long bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
DEV uint32_t lds_addr(const void* p) { return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p; }

// Fragment reads are inline asm: the compiler's wait-count insertion would otherwise order every LDS
// read after ALL outstanding direct-to-LDS loads (it cannot tell the pipeline stages apart) and
// serialise the pipeline.  The caller waits with lds_wait_* below, which ties the registers to the wait.
template <int OFF>
DEV u32x4 ds_read_b128_at(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
DEV u32x2 ds_read_tr_at(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

// per-lane byte offset (inside a KC tile) of the fragment chunk (row lane%32, chunk 2 ks + lane/32);
// rows 32 j further on add 2048 j bytes
DEV uint32_t kc_frag_off(int lane, int ks) {
  const int fr = lane & 31, kc = 2 * ks + (lane >> 5);
  return (uint32_t)((fr * 4 + (kc ^ ((fr >> 2) & 3))) << 4);
}
// per-lane byte offset (inside a KS tile of R rows) of the first of the two transposing reads of the
// fragment (rows n0 .. n0+31, n0 % 32 == 0, contraction 16 ks + 8 (lane/32) ..); the second read is
// 4 k rows (8 R bytes) further.  tile_n32 = n0 / 32.
template <int R>
DEV uint32_t ks_frag_off(int lane, int ks, int tile_n32) {
  const int s = lane & 15, nh = (lane >> 4) & 1, kh = lane >> 5;
  const int n = 16 * nh + 4 * (s & 3);
  const int k = 16 * ks + 8 * kh + (s >> 2);
  return (uint32_t)(k * (R * 2) + ((tile_n32 ^ (k & 3)) << 6) + n * 2);
}

struct IdentityCols {
  int row0, row_end;
  DEV int operator()(int r) const { int g = row0 + r; return g < row_end ? g : -1; }
};

// Issues the loads of one operand tile.  R rows, NW waves in the workgroup; each wave owns IPW of the
// tile's R/16 one-KiB pieces.
template <int R, int NW, bool KS>
struct DmaLoader {
  static_assert(R % (16 * NW) == 0, "tile pieces must divide over the waves");
  static constexpr int IPW = R / 16 / NW;
  uint32_t base[IPW];   // byte offset of the lane's chunk at k0 = 0, or BUF_OOB
  int kofs;             // KC: contraction offset of the lane's chunk inside the tile (K-tail test)
  int ld2;              // KS: bytes per memory row

  // KC: memory [row][k]; rows row0.. clipped at row_end.
  DEV void init_kc(int ld, int row0, int row_end, int wave, int lane) {
    const int kc = (lane & 3) ^ ((lane >> 4) & 3);
    kofs = kc * 8;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int r = row0 + 16 * (wave * IPW + i) + (lane >> 2);
      base[i] = r < row_end ? (uint32_t)(r * ld + kofs) * 2u : BUF_OOB;
    }
  }
  // KS: memory [k][row]; cols(r) maps a tile-local row (multiple of 8) to its memory column or -1.
  // Contraction indices past the operand's last memory row fall outside the buffer extent by themselves.
  template <class ColMap>
  DEV void init_ks(int ld, const ColMap& cols, int wave, int lane) {
    ld2 = ld * 2;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int P = (wave * IPW + i) * 1024 + lane * 16;
      const int k = P / (R * 2), w = P % (R * 2);
      const int g = (w >> 6) ^ (k & 3), sub = (w >> 4) & 3;
      const int c = cols(g * 32 + sub * 8);
      base[i] = c >= 0 ? (uint32_t)(k * ld + c) * 2u : BUF_OOB;
    }
  }
  // extra: a wave-uniform byte offset added to in-range lanes (e.g. a row offset of a KC operand)
  DEV void issue(buf_rsrc rs, uint8_t* tile, int k0, int k_end, int wave, uint32_t extra = 0) const {
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      uint32_t off;
      if (KS) off = base[i] + (uint32_t)(k0 * ld2) + extra;
      else off = (k0 + kofs < k_end) ? base[i] + (uint32_t)k0 * 2u + extra : BUF_OOB;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, LDS_PTR(tile + (wave * IPW + i) * 1024), 16, off, 0, 0, 0);
    }
  }
};

// Explicit LDS waits for the asm reads: lds_wait<N>() returns once at most N LDS operations of this wave
// are outstanding (they complete in order); tie() makes a register "used and redefined" after the wait
// so that no consumer can be scheduled above it.
template <int N>
DEV void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
DEV void tie(u32x4& v) { asm volatile("" : "+v"(v)); }
DEV void tie(u32x2& v) { asm volatile("" : "+v"(v)); }

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14; expcnt, lgkmcnt left open)
template <int N>
DEV void wait_vmcnt() { __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70); }
