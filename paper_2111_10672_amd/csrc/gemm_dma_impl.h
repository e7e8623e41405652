// bfloat16 products on the gfx950 matrix cores with direct-to-LDS operand loads.
//
//   C[m, n] = sum_k A(m, k) * B(n, k),   float32 accumulation
//
// Same three products as gemm.hip (forward, input gradient, weight gradient of a dense layer), built
// around two CDNA4 facilities:
//   * global_load_lds_dwordx4: every lane fetches 16 bytes from its own global address and the wave's
//     64 chunks land in one contiguous KiB of LDS, without passing through registers.  Several tiles
//     can therefore be in flight at once (STAGES-deep ring); which chunk a lane fetches is chosen so
//     that the KiB it fills is already in the bank-friendly order the matrix-core reads want.
//   * ds_read_b64_tr_b16: a transposing LDS read.  An operand whose *row* index is contiguous in memory
//     (the layout of both weight-gradient operands and of W in the input-gradient product) is copied to
//     LDS as it lies and transposed on the way to the registers.  Within 16 lanes, lane j receives
//     element (j % 4) of the 8-byte words read by lanes j/4, j/4 + 4, j/4 + 8, j/4 + 12; pointing lane j'
//     at 4 consecutive rows starting at row 4 * (j' % 4) of k-row j'/4 gives lane j four consecutive k
//     of row j, which is the MFMA operand layout.
// Tile loop: wait for tile t (s_waitcnt vmcnt leaves the younger tiles' loads in flight), one barrier,
// issue tile t + STAGES - 1 into the buffer tile t - 1 used, multiply tile t.
#pragma once
#include <type_traits>
#include "gemm_common.h"

namespace spb {
namespace gemm_dma_detail {
using namespace gemm_detail;

__device__ __forceinline__ long long batch_offset_z(const BatchStride& b, int z) { return z == 0 ? 0 : batch_offset(b, z); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* global_ptr_t;

static __device__ const uint32_t kZeroChunk[4] = {0u, 0u, 0u, 0u};

constexpr int kTileK = 64;  // bfloat16 elements of k per tile: 128 bytes per row

// s_waitcnt immediate for gfx9: vmcnt in bits 3:0 and 15:14, expcnt 6:4 (7 = no wait), lgkmcnt 11:8.
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 15) << 8); }

template <int VM>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(VM, 0));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Rotation (in 16-byte chunks) of k-row k of a KRow tile, so that the four k-rows one transposing read
// touches fall into different 64-byte bank groups.
// A k-row is ROWS * 2 bytes, so where consecutive k-rows start (mod the 256 bytes of the banks) depends on ROWS:
// a multiple of 256 bytes (ROWS = 128, 256): every k-row starts in the same place and k-row k is rotated by k % 4
// groups; an odd multiple of 128 bytes (ROWS = 64, 192): k-rows already alternate between the two halves, and the
// rotation only has to separate k from k + 2.  (With ROWS = 192 the first rule sends k and k + 2 to the same
// banks wherever the rotation wraps around the row.)
template <int ROWS>
__device__ __forceinline__ int krow_rot(int k) {
  if constexpr ((ROWS * 2) % 256 == 0) return (k & 3) << 2;
  else if constexpr ((ROWS * 2) % 256 == 128) return ((k >> 1) & 1) << 2;
  else return 0;
}

// Where one lane's 16-byte chunks of an operand tile come from.  Everything that does not change from
// tile to tile is worked out once; tiles are issued in increasing order, so what does change (the tap and
// channel a chunk's k falls on, the pixel a k-row stands for) is stepped, never divided out again.
// Every wave issues exactly kInstr direct-to-LDS instructions per tile, whatever its lanes' predicates, so
// the vmcnt arithmetic of the tile loop holds: a lane whose k lies beyond K (or, gathered operands, whose pixel
// lies in the zero padding or beyond the tensor) fetches a chunk of zeros instead.
template <int ROWS, Layout L, Gather G, int NW>
struct TileSource {
  static constexpr int kInstr = ROWS / (8 * NW);
  static_assert(ROWS % (8 * NW) == 0 && kInstr >= 1, "tile rows must fill whole wave instructions");
  static_assert(G == Gather::None || (G == Gather::ConvRows) == (L == Layout::RowK), "gather kind fixes the LDS layout");
  const char* ptr[kInstr];  // Gathers: the tensor's base (or, one tap per tile, this lane's pixel at tap (0, 0)).
  int k_in_tile[kInstr];    // k of the chunk's first element relative to the tile start
  bool in_rows[kInstr];
  int row_idx[kInstr];      // first row (of the operand) this lane's chunk covers
  size_t tile_step;         // Plain: bytes from one tile to the next
  // Plain operands: a chunk's address is a wave-uniform panel address, stepped from tile to tile with scalar
  // arithmetic, plus a 32-bit lane offset that never changes.  Rows beyond the matrix are not redirected to zeros:
  // their offset is clamped onto the last rows of the matrix, whose values then fill result rows (or columns) that
  // no epilogue stores.  Only k beyond K must multiply as zero, and only the last tile can contain such k.
  const char* panel;        // tile t_first of this workgroup's rows
  uint32_t voff[kInstr];
  int t_first;
  // gather state, per instruction
  int tap[kInstr], chan[kInstr];           // ConvRows, ConvWeightT: where this lane's k of the next tile falls; ConvPatchT: fixed (tap, ci) of its rows
  int g0[kInstr], g1[kInstr], g2[kInstr];  // ConvRows: pixel base, row term, column term.  ConvPatchT: image, pixel in image of the next tile's k-row.
  int step_q, step_r;                      // one tile further: quotient and remainder of 64 by the modulus being stepped
  // ConvRows whose channel count is a multiple of the tile's k (and, transposed, stride 1): a whole tile lies on
  // ONE tap, so the tap and its offset are wave-uniform scalars and a lane only adds them to the address of its
  // pixel (ptr[] then holds that address, at tap (0, 0)) and checks its two coordinates.
  bool one_tap;
  int u_tap, u_chan;

  __device__ __forceinline__ void init(const bf16_t* base, int ld, int row0, int nrows, int wave, int lane, int t0, const ConvGeom& cg) {
    tile_step = L == Layout::RowK ? (size_t)kTileK * 2 : (size_t)kTileK * ld * 2;
    const int modulus = G == Gather::ConvRows ? cg.sc : G == Gather::ConvWeightT ? cg.w_cout : cg.rh * cg.rw;
    if constexpr (G != Gather::None) { step_q = kTileK / modulus; step_r = kTileK % modulus; }
    one_tap = false;
    if constexpr (G == Gather::ConvRows) {
      one_tap = cg.sc % kTileK == 0 && (!cg.transposed || cg.stride == 1);
      u_tap = (t0 * kTileK) / cg.sc; u_chan = (t0 * kTileK) % cg.sc;
    }
#pragma unroll
    for (int i = 0; i < kInstr; ++i) {
      const int slot = (i * NW + wave) * 64 + lane;
      int gr, k;
      if constexpr (L == Layout::RowK) {
        const int row = slot >> 3, pc = slot & 7;
        gr = row0 + row;
        k = ((pc ^ row ^ ((row >> 3) & 3)) & 7) << 3;   // the inverse of lds_offset
      } else {
        constexpr int kRowChunks = ROWS / 8;
        k = slot / kRowChunks;
        const int pc = slot % kRowChunks;
        gr = row0 + (((pc - krow_rot<ROWS>(k) + kRowChunks) % kRowChunks) << 3);
      }
      k_in_tile[i] = k;
      in_rows[i] = gr < nrows;
      row_idx[i] = gr;
      if constexpr (G == Gather::None) {
        t_first = t0;
        if constexpr (L == Layout::RowK) {
          panel = reinterpret_cast<const char*>(base + (size_t)row0 * ld) + (size_t)t0 * tile_step;
          voff[i] = (uint32_t)(min(gr, nrows - 1) - row0) * (uint32_t)ld * 2u + (uint32_t)k * 2u;
        } else {
          panel = reinterpret_cast<const char*>(base) + (size_t)t0 * tile_step;
          voff[i] = (uint32_t)k * (uint32_t)ld * 2u + (uint32_t)(gr < nrows ? gr : ((nrows - 1) & ~7)) * 2u;   // a chunk is 8 rows
        }
      } else {
        ptr[i] = reinterpret_cast<const char*>(base);
        const int k_abs = t0 * kTileK + k;
        if constexpr (G == Gather::ConvRows) {        // row gr = pixel (n, a, b); k = (tap, channel)
          const int per_image = cg.rh * cg.rw;
          const int n = gr / per_image, rem = gr - n * per_image;
          const int a = rem / cg.rw, b = rem - a * cg.rw;
          g0[i] = n * cg.sh * cg.sw;
          g1[i] = cg.transposed ? a + cg.pad : a * cg.stride - cg.pad;
          g2[i] = cg.transposed ? b + cg.pad : b * cg.stride - cg.pad;
          tap[i] = k_abs / cg.sc; chan[i] = k_abs - tap[i] * cg.sc;
          if (one_tap) ptr[i] += ((long long)(g0[i] + g1[i] * cg.sw + g2[i]) * cg.sc + k) * 2;
        } else if constexpr (G == Gather::ConvWeightT) {  // row gr = ci; k = (tap, co)
          tap[i] = k_abs / cg.w_cout; chan[i] = k_abs - tap[i] * cg.w_cout;
        } else {                                          // row gr = (tap, ci); k = output pixel m
          tap[i] = gr / cg.sc; chan[i] = gr - tap[i] * cg.sc;
          const int per_image = cg.rh * cg.rw;
          g0[i] = k_abs / per_image; g1[i] = k_abs - g0[i] * per_image; g2[i] = 0;
        }
      }
    }
  }

  // Issue tile t (tiles must be issued in increasing order, one after the other).  PARTS > 1: only the
  // instructions i with i % PARTS == part, and the parts of a tile in increasing order.
  template <int PARTS = 1>
  __device__ __forceinline__ void issue(int t, int K, char* tile, int wave, int ld, const ConvGeom& cg, int part = 0) {
    if constexpr (G == Gather::ConvRows) {
      if (one_tap) {
        const int r = (u_tap * (65536 / cg.s + 1)) >> 16, c = u_tap - r * cg.s;   // tap = r * S + c, exact for tap < 256
        const int dr = cg.transposed ? -r : r, dc = cg.transposed ? -c : c;
        const long long tap_bytes = ((long long)(dr * cg.sw + dc) * cg.sc + u_chan) * 2;
        const bool tap_ok = u_tap < cg.r * cg.s;
#pragma unroll
        for (int i = 0; i < kInstr; ++i) {
          if (PARTS > 1 && i % PARTS != part) continue;
          const bool ok = tap_ok && in_rows[i] && (unsigned)(g1[i] + dr) < (unsigned)cg.sh && (unsigned)(g2[i] + dc) < (unsigned)cg.sw;
          const char* src = ok ? ptr[i] + tap_bytes : reinterpret_cast<const char*>(kZeroChunk);
          __builtin_amdgcn_global_load_lds((global_ptr_t)src, (lds_ptr_t)(tile + (i * NW + wave) * 1024), 16, 0, 0);
        }
        if (part == PARTS - 1) {   // the tile is complete: on to the next tap or channel block
          u_chan += kTileK;
          if (u_chan >= cg.sc) { u_chan = 0; ++u_tap; }
        }
        return;
      }
    }
    if constexpr (G == Gather::None) {
      const char* pt = panel + (size_t)(t - t_first) * tile_step;      // uniform over the wave
      if ((t + 1) * kTileK <= K) {                                     // a whole tile: no lane has anything to check
        // Written as assembly to get the scalar-base form (address = SGPR pair + 32-bit lane offset): through the
        // builtin the compiler keeps a 64-bit pointer per instruction in VGPRs, steps each with vector adds and
        // folds this branch into per-lane selects, a dozen vector instructions per load that compete with the
        // MFMAs for issue.  M0 holds the LDS address of the KiB the wave's 64 chunks fill.
#pragma unroll
        for (int i = 0; i < kInstr; ++i) {
          if (PARTS > 1 && i % PARTS != part) continue;
          const uint32_t dst = (uint32_t)(uintptr_t)(lds_ptr_t)(tile + (i * NW + wave) * 1024);
          asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff[i]), "s"(pt), "s"(dst) : "m0");
        }
      } else {                                                         // the last tile of a k range that ends inside it
#pragma unroll
        for (int i = 0; i < kInstr; ++i) {
          if (PARTS > 1 && i % PARTS != part) continue;
          const char* src = t * kTileK + k_in_tile[i] < K ? pt + voff[i] : reinterpret_cast<const char*>(kZeroChunk);
          __builtin_amdgcn_global_load_lds((global_ptr_t)src, (lds_ptr_t)(tile + (i * NW + wave) * 1024), 16, 0, 0);
        }
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < kInstr; ++i) {
      if (PARTS > 1 && i % PARTS != part) continue;
      const char* src = reinterpret_cast<const char*>(kZeroChunk);
      if constexpr (G == Gather::None) {
      } else if constexpr (G == Gather::ConvRows) {
        const int taps = cg.r * cg.s;
        const int r = (tap[i] * (65536 / cg.s + 1)) >> 16, c = tap[i] - r * cg.s;   // tap = r * S + c, exact for tap < 256
        int hi, wi;
        bool ok = in_rows[i] && tap[i] < taps;
        if (!cg.transposed) {
          hi = g1[i] + r; wi = g2[i] + c;
        } else {
          const int th = g1[i] - r, tw = g2[i] - c, m = cg.stride - 1;   // stride is 1 or 2
          ok = ok && th >= 0 && tw >= 0 && ((th | tw) & m) == 0;
          hi = th >> m; wi = tw >> m;
        }
        ok = ok && (unsigned)hi < (unsigned)cg.sh && (unsigned)wi < (unsigned)cg.sw;
        if (ok) src = ptr[i] + ((size_t)(g0[i] + hi * cg.sw + wi) * cg.sc + chan[i]) * 2;
        chan[i] += step_r; tap[i] += step_q;
        if (chan[i] >= cg.sc) { chan[i] -= cg.sc; ++tap[i]; }
      } else if constexpr (G == Gather::ConvWeightT) {
        const int taps = cg.r * cg.s;
        if (in_rows[i] && tap[i] < taps) src = ptr[i] + (((size_t)chan[i] * taps + tap[i]) * cg.w_cin + row_idx[i]) * 2;
        chan[i] += step_r; tap[i] += step_q;
        if (chan[i] >= cg.w_cout) { chan[i] -= cg.w_cout; ++tap[i]; }
      } else {
        const int r = (tap[i] * (65536 / cg.s + 1)) >> 16, c = tap[i] - r * cg.s;
        const int oh = __float2int_rz(((float)g1[i] + 0.5f) * (1.0f / (float)cg.rw)), ow = g1[i] - oh * cg.rw;
        const int hi = oh * cg.stride + r - cg.pad, wi = ow * cg.stride + c - cg.pad;
        if (in_rows[i] && g0[i] < cg.n && (unsigned)hi < (unsigned)cg.sh && (unsigned)wi < (unsigned)cg.sw)
          src = ptr[i] + ((size_t)((g0[i] * cg.sh + hi) * cg.sw + wi) * cg.sc + chan[i]) * 2;
        const int per_image = cg.rh * cg.rw;
        g1[i] += step_r; g0[i] += step_q;
        if (g1[i] >= per_image) { g1[i] -= per_image; ++g0[i]; }
      }
      __builtin_amdgcn_global_load_lds((global_ptr_t)src, (lds_ptr_t)(tile + (i * NW + wave) * 1024), 16, 0, 0);
    }
  }

};

// Fetch the MFMA operand of one 32-row fragment for k-group kg (16 values of k): 8 bfloat16 per lane.
// A KRow fragment is read in assembly and is valid only after fragments_ready().
template <int ROWS, Layout L>
__device__ __forceinline__ u32x4 read_fragment(const char* tile, int frag_row0, int kg, int lane) {
  if constexpr (L == Layout::RowK) {
    return *reinterpret_cast<const u32x4*>(tile + lds_offset(frag_row0 + (lane & 31), 2 * kg + (lane >> 5)));
  } else {
    constexpr int kRowChunks = ROWS / 8;
    const int j = lane & 15, g = lane >> 4;
    const int row = frag_row0 + 16 * (g & 1) + 4 * (j & 3);  // first of the 4 rows this lane's word covers
    u32x4 out;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k = 16 * kg + 8 * (g >> 1) + 4 * h + (j >> 2);
      const int pc = ((row >> 3) + krow_rot<ROWS>(k)) % kRowChunks;
      const char* addr = tile + k * (ROWS * 2) + pc * 16 + (row & 7) * 2;
      // Written as assembly: through the builtin the compiler cannot tell this read from the in-flight
      // direct-to-LDS tiles and drains them all (vmcnt 0) first.
      const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)addr;
      uint2 w;
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(w) : "v"(lds_addr));
      out[2 * h] = w.x;
      out[2 * h + 1] = w.y;
    }
    return out;
  }
}

// Wait for the LDS reads issued in assembly and pin every later use of the fragments behind the wait.
template <int NA, int NB>
__device__ __forceinline__ void fragments_ready(u32x4 (&a)[NA], u32x4 (&b)[NB]) {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < NA; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
  for (int j = 0; j < NB; ++j) asm volatile("" : "+v"(b[j]));
}

// The same fetch with every LDS read written as assembly, for the loop that keeps direct-to-LDS loads in flight
// across its LDS reads on purpose: nothing here lets the compiler tie a read to those loads and wait for them,
// and the reads stay in source order.  Valid after an s_waitcnt lgkmcnt and a pin (fragments_ready, pin_fragment).
__device__ __forceinline__ u32x4 lds_read_b128_asm(const char* addr) {
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)addr;
  u32x4 w;
  asm volatile("ds_read_b128 %0, %1" : "=v"(w) : "v"(lds_addr));
  return w;
}
template <int ROWS, Layout L>
__device__ __forceinline__ u32x4 read_fragment_asm(const char* tile, int frag_row0, int kg, int lane) {
  if constexpr (L == Layout::RowK) return lds_read_b128_asm(tile + lds_offset(frag_row0 + (lane & 31), 2 * kg + (lane >> 5)));
  else return read_fragment<ROWS, L>(tile, frag_row0, kg, lane);
}

// MFMA operand reads with every lane-dependent part of the address worked out once.  For a RowK tile the lane part
// depends on the k-group (the chunk permutation is an XOR) but not on the fragment: 4 offsets, fragment i adds
// i * 32 rows as an instruction offset.  For a KRow tile it depends on the fragment (where the rotation wraps
// around the row) but not on the k-group: T offsets, k-group kg and half h add (16 kg + 4 h) k-rows as an
// instruction offset.  at(tile) adds a tile's LDS address to them: one vector add each per tile instead of
// one or two per read.
template <int ROWS, Layout L, int T>
struct FragmentReader {
  static constexpr int kN = L == Layout::RowK ? 4 : T;
  uint32_t off[kN];
  __device__ __forceinline__ void init(int wave_row0, int lane) {   // wave_row0: a multiple of 32
    if constexpr (L == Layout::RowK) {
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) off[kg] = (uint32_t)lds_offset(wave_row0 + (lane & 31), 2 * kg + (lane >> 5));
    } else {
      constexpr int kRowChunks = ROWS / 8;
      const int j = lane & 15, g = lane >> 4;
#pragma unroll
      for (int i = 0; i < T; ++i) {
        const int row = wave_row0 + 32 * i + 16 * (g & 1) + 4 * (j & 3);
        const int k = 8 * (g >> 1) + (j >> 2);                    // 16 kg + 4 h is a multiple of 4: it leaves the rotation alone
        const int pc = ((row >> 3) + krow_rot<ROWS>(k)) % kRowChunks;
        off[i] = (uint32_t)(k * (ROWS * 2) + pc * 16 + (row & 7) * 2);
      }
    }
  }
  __device__ __forceinline__ void at(uint32_t tile_lds_address, uint32_t (&out)[kN]) const {
#pragma unroll
    for (int n = 0; n < kN; ++n) out[n] = off[n] + tile_lds_address;
  }
  // fragment I, k-group KG of the tile whose addresses are `a`; valid after an s_waitcnt lgkmcnt and a pin
  template <int I, int KG>
  static __device__ __forceinline__ u32x4 read(const uint32_t (&a)[kN]) {
    u32x4 out;
    if constexpr (L == Layout::RowK) {
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(out) : "v"(a[KG]), "n"(I * 32 * kRowBytes));
    } else {
      uint2 lo, hi;
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a[I]), "n"((16 * KG) * (ROWS * 2)));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a[I]), "n"((16 * KG + 4) * (ROWS * 2)));
      out[0] = lo.x; out[1] = lo.y; out[2] = hi.x; out[3] = hi.y;
    }
    return out;
  }
};

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) { return bf16_pack2(lo, hi); }

// Epilogue.  Each wave parks 32 rows of its WM x WN accumulator tile at a time in its own LDS region (the tile
// ring is dead by then) and reads them back row by row, so that bias, mask and result move in 16-byte pieces
// along n.  LDS operations of one wave complete in order, so the pieces need no barrier between them.
// The row loops are deliberately not unrolled: an unrolled epilogue is tens of thousands of instructions,
// which no longer fit the instruction cache and cost more time than the tile loop itself.

// All bfloat16 epilogues are one formula per element,
//     out = act(alpha * acc * s + b + r),
// with s, b per column and r per element:  BiasAct: s = column scale or 1, b = bias or 0, r = residual or 0;
// MaskStore: s = [x > 0]; ScaleStore: s = x, where x is the per-element tensor `mask`.  At most one
// per-element tensor is read (residual or mask), so a unit of 8 outputs costs one optional 16-byte global load,
// which is fetched one unit ahead of its use.

__device__ __forceinline__ void unpack_bf16x8(const u32x4& w, float (&f)[8]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) { f[2 * d] = __uint_as_float(w[d] << 16); f[2 * d + 1] = __uint_as_float(w[d] & 0xFFFF0000u); }
}
__device__ __forceinline__ u32x4 pack_bf16x8(const float (&f)[8]) {
  u32x4 o;
#pragma unroll
  for (int d = 0; d < 4; ++d) o[d] = pack_bf16(f[2 * d], f[2 * d + 1]);
  return o;
}

// ragged right edge: the last, partly filled group of columns, element by element, straight from the parked row
__device__ __forceinline__ void store_ragged(const GemmParams& p, const float* parked, int count, int m, int n, long long c_offset) {
  const bf16_t* bias = static_cast<const bf16_t*>(p.bias);
  if (p.epilogue == (int)Epilogue::StoreF32) {
    float* dst = static_cast<float*>(p.C) + c_offset + (size_t)m * p.ldc + n;
#pragma unroll 1
    for (int e = 0; e < count && n + e < p.N; ++e) dst[e] = parked[e] * p.alpha + (bias ? to_float(bias[n + e]) : 0.f);
    return;
  }
  const bf16_t* mask = static_cast<const bf16_t*>(p.mask);
  const bf16_t* res = static_cast<const bf16_t*>(p.residual);
  const bf16_t* cscale = static_cast<const bf16_t*>(p.col_scale);
  bf16_t* aux = static_cast<bf16_t*>(p.aux_out);
  bf16_t* dst = static_cast<bf16_t*>(p.C) + c_offset + (size_t)m * p.ldc + n;
#pragma unroll 1
  for (int e = 0; e < count && n + e < p.N; ++e) {
    float v = parked[e] * p.alpha, pre = v;
    if (p.epilogue == (int)Epilogue::MaskStore) v = to_float(mask[(size_t)m * p.ldmask + n + e]) > 0.f ? v : 0.f;
    else if (p.epilogue == (int)Epilogue::ScaleStore) v *= to_float(mask[(size_t)m * p.ldmask + n + e]);
    else {
      v = v * (cscale ? to_float(cscale[n + e]) : 1.f) + (bias ? to_float(bias[n + e]) : 0.f);
      if (!p.aux_raw) pre = v;
      if (res) v += to_float(res[(size_t)m * p.ldres + n + e]);
      if (p.act == (int)Act::Relu) v = fmaxf(v, 0.f);
      else if (p.act == (int)Act::Gelu) {
        if (p.aux_act_grad) gelu_both_f(v, v, pre);
        else v = gelu_f(v);
      }
      if (aux) store_elem(aux + (size_t)m * p.ldaux + n + e, pre);
    }
    store_elem(dst + e, v);
  }
}

// Per-column operands of the bfloat16 epilogue for the 8 columns a lane owns: loaded once per wave tile, and by
// the small-product kernel before its tile loop so that their latency is not paid at the end.
struct ColumnOperands {
  u32x4 sc, bs;  // 8 bfloat16 each, unpacked where they are used so that requesting them early waits for nothing
};
template <int WN>
__device__ __forceinline__ void load_column_operands(const GemmParams& p, int col_base, int lane, ColumnOperands& o) {
  const int n = col_base + (lane % (WN / 8)) * 8;
  o.sc = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};  // ones
  o.bs = u32x4{0u, 0u, 0u, 0u};
  if (p.epilogue != (int)Epilogue::BiasAct || n + 8 > p.N) return;
  if (p.col_scale) o.sc = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.col_scale) + n);
  if (p.bias) o.bs = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.bias) + n);
}

// The per-element tensor of the bfloat16 epilogue (residual or mask) for the first two rows a lane owns: what the
// small-product kernel, whose waves finish at most 16 rows each, requests before its tile loop.
template <int WN>
__device__ __forceinline__ void load_row_operands(const GemmParams& p, int piece_row, int col_base, int lane, u32x4 (&x)[2]) {
  constexpr int kPerRow = WN / 8, kRowStep = 64 / kPerRow;
  const int n = col_base + (lane % kPerRow) * 8;
  const bool plain = p.epilogue == (int)Epilogue::BiasAct;
  const bf16_t* xsrc = plain ? static_cast<const bf16_t*>(p.residual) : static_cast<const bf16_t*>(p.mask);
  const int ldx = plain ? p.ldres : p.ldmask;
  x[0] = u32x4{0u, 0u, 0u, 0u};
  x[1] = x[0];
  if (p.epilogue == (int)Epilogue::StoreF32 || xsrc == nullptr || n + 8 > p.N) return;
#pragma unroll
  for (int it = 0; it < 2; ++it)
    x[it] = *reinterpret_cast<const u32x4*>(xsrc + (size_t)min(piece_row + lane / kPerRow + it * kRowStep, p.M - 1) * ldx + n);
}

// The row loops read PARTS partial tiles, part_stride floats apart, and add them up (one tile for the large
// kernels, the four waves' partial sums for the small-product kernel).
template <int WN, int PARTS = 1>
__device__ __forceinline__ void store_rows_f32(const GemmParams& p, const float* stage, int piece_row, int col_base, int lane, long long c_offset,
                                               int rows = 32, int part_stride = 0) {
  constexpr int kPitch = WN + 4;
  constexpr int kPerRow = WN / 4;             // 4-column units per row; a lane's column never changes
  constexpr int kRowStep = 64 / kPerRow;      // rows per pass; with 96 columns the last lanes of the wave sit out
  const int c = (lane % kPerRow) * 4, n = col_base + c;
  if (n >= p.N || lane >= kPerRow * kRowStep) return;
  const bool whole = n + 4 <= p.N;
  f32x4 b = {0.f, 0.f, 0.f, 0.f};
  if (p.bias && whole) {
    const uint2 bb = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(p.bias) + n);
    b[0] = __uint_as_float(bb.x << 16); b[1] = __uint_as_float(bb.x & 0xFFFF0000u);
    b[2] = __uint_as_float(bb.y << 16); b[3] = __uint_as_float(bb.y & 0xFFFF0000u);
  }
#pragma unroll 1
  for (int row = lane / kPerRow; row < rows; row += kRowStep) {
    const int m = piece_row + row;
    if (m >= p.M) break;
    f32x4 v = *reinterpret_cast<const f32x4*>(stage + row * kPitch + c);
#pragma unroll
    for (int w = 1; w < PARTS; ++w) v += *reinterpret_cast<const f32x4*>(stage + w * part_stride + row * kPitch + c);
    if (whole) {
      *reinterpret_cast<f32x4*>(static_cast<float*>(p.C) + c_offset + (size_t)m * p.ldc + n) = v * p.alpha + b;
    } else {
      float t[4] = {v[0], v[1], v[2], v[3]};
      store_ragged(p, t, 4, m, n, c_offset);
    }
  }
}

template <int WN, int PARTS = 1>
__device__ __forceinline__ void store_rows_bf16(const GemmParams& p, const float* stage, int piece_row, int col_base, int lane, long long c_offset,
                                                int rows = 32, int part_stride = 0, const ColumnOperands* preloaded = nullptr,
                                                const u32x4* xpre = nullptr) {
  constexpr int kPitch = WN + 4;
  constexpr int kPerRow = WN / 8;             // 8-column units per row; a lane's column never changes
  constexpr int kRowStep = 64 / kPerRow;      // rows per pass; with 96 columns the last lanes of the wave sit out
  const int c = (lane % kPerRow) * 8, n = col_base + c;
  if (n >= p.N || lane >= kPerRow * kRowStep) return;
  const int mode = p.epilogue;
  const bool plain = mode == (int)Epilogue::BiasAct;
  bf16_t* aux = plain ? static_cast<bf16_t*>(p.aux_out) : nullptr;
  // the per-element tensor this epilogue reads, if any
  const bf16_t* xsrc = plain ? static_cast<const bf16_t*>(p.residual) : static_cast<const bf16_t*>(p.mask);
  const int ldx = plain ? p.ldres : p.ldmask;
  if (n + 8 > p.N) {
#pragma unroll 1
    for (int row = lane / kPerRow; row < rows && piece_row + row < p.M; row += kRowStep) {
      float t[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        t[e] = stage[row * kPitch + c + e];
#pragma unroll
        for (int w = 1; w < PARTS; ++w) t[e] += stage[w * part_stride + row * kPitch + c + e];
      }
      store_ragged(p, t, 8, piece_row + row, n, c_offset);
    }
    return;
  }
  ColumnOperands cols;
  if (preloaded) cols = *preloaded;
  else load_column_operands<WN>(p, col_base, lane, cols);
  float sc[8], bs[8];
  unpack_bf16x8(cols.sc, sc);
  unpack_bf16x8(cols.bs, bs);
  // One unit: 8 outputs of row `row` from the parked accumulators and the per-element tensor's chunk xcur.
  auto unit = [&](int row, int m, const u32x4& xcur) {
    float v[8], x[8], pre[8];
    f32x4 v0 = *reinterpret_cast<const f32x4*>(stage + row * kPitch + c);
    f32x4 v1 = *reinterpret_cast<const f32x4*>(stage + row * kPitch + c + 4);
#pragma unroll
    for (int w = 1; w < PARTS; ++w) {
      v0 += *reinterpret_cast<const f32x4*>(stage + w * part_stride + row * kPitch + c);
      v1 += *reinterpret_cast<const f32x4*>(stage + w * part_stride + row * kPitch + c + 4);
    }
    unpack_bf16x8(xcur, x);
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = v0[e] * p.alpha; v[4 + e] = v1[e] * p.alpha; }
    if (mode == (int)Epilogue::MaskStore) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = x[e] > 0.f ? v[e] : 0.f;
    } else if (mode == (int)Epilogue::ScaleStore) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] *= x[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pre[e] = v[e];
        v[e] = v[e] * sc[e] + bs[e];
        if (!p.aux_raw) pre[e] = v[e];
        v[e] += x[e];                           // a residual joins before the activation (residual blocks); x = 0 without one
      }
      if (p.act == (int)Act::Relu) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
      } else if (p.act == (int)Act::Gelu) {
        if (p.aux_act_grad) {
#pragma unroll
          for (int e = 0; e < 8; ++e) gelu_both_f(v[e], v[e], pre[e]);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
        }
      }
      if (aux) *reinterpret_cast<u32x4*>(aux + (size_t)m * p.ldaux + n) = pack_bf16x8(pre);
    }
    *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.C) + c_offset + (size_t)m * p.ldc + n) = pack_bf16x8(v);
  };
  const int row0 = lane / kPerRow;
  if (xpre) {              // at most two rows per lane, their chunks already requested (see load_row_operands)
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int row = row0 + it * kRowStep;
      if (row < rows && piece_row + row < p.M) unit(row, piece_row + row, xpre[it]);
    }
    return;
  }
  if (xsrc == nullptr) {   // nothing to read per element: stores only, nothing to wait for
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll 1
    for (int row = row0; row < rows && piece_row + row < p.M; row += kRowStep) unit(row, piece_row + row, zero);
    return;
  }
  // The tensor's chunk for the next unit is requested (from a clamped, always valid row) before this unit's
  // stores are issued, so waiting for it never waits for a store.
  const int last_row = p.M - 1;
  u32x4 xnext = *reinterpret_cast<const u32x4*>(xsrc + (size_t)min(piece_row + row0, last_row) * ldx + n);
#pragma unroll 1
  for (int row = row0; row < rows && piece_row + row < p.M; row += kRowStep) {
    const int m = piece_row + row;
    const u32x4 xcur = xnext;
    xnext = *reinterpret_cast<const u32x4*>(xsrc + (size_t)min(m + kRowStep, last_row) * ldx + n);
    unit(row, m, xcur);
  }
}

// Epilogue of the large kernels.  Their tile loops multiply with the operands exchanged (the N-side fragment is the
// MFMA's first operand), so the 16 accumulators a lane holds of a 32 x 32 block are 16 columns of ONE output row:
// row = lane % 32, column = 8 * (r / 4) + 4 * (lane / 32) + r % 4.  Four consecutive registers are four consecutive
// columns, so a wave parks 32 rows of its tile in its own LDS region (the tile ring is dead by then) with one
// 16-byte write per four accumulators, and reads them back so that consecutive lanes hold consecutive 16-byte
// pieces of a row: loads of the per-element tensor and stores of the result are whole 64-byte segments per four
// lanes (stores scattered one lane per row were measured 2-3 x slower: every lane becomes a request of its own at the
// L2).  LDS operations of one wave complete in order, so no barrier separates the pieces.  A wave issues about 1.7 k
// instructions at 4 cycles each if this is written as a loop over rows with the mode tested per element (8 us per
// product, as much as 12 k-tiles of the tile loop); hence: the row loop is unrolled with the mode decided outside
// it, a lane's column and its per-column operands never change, a row's address is the previous one plus a constant,
// and the per-element chunks of the next 32 rows are requested before the current ones are stored, so waiting for
// them never waits for a store.  The arithmetic per element is that of store_rows_bf16.
// wm, tile_m: the wave's place among the WAVES_M waves that share its columns and the tile's row of tiles (the fused
// affine backward adds its column sums up over those waves and files them under that row).
template <int WM, int WN, int WAVES_M>
__device__ __forceinline__ void store_wave_tile(const GemmParams& p, f32x16 (&acc)[WM / 32][WN / 32], float* stage, int row_base, int col_base, int lane, long long c_offset,
                                                int wm, int tile_m) {
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kPitch = WN + 4;  // floats; the 16-byte pad staggers the banks of consecutive rows
  float* park_at = stage + (lane & 31) * kPitch + 4 * (lane >> 5);
  auto park = [&](int i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<f32x4*>(park_at + j * 32 + 8 * g) = f32x4{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
  };
  if (p.epilogue == (int)Epilogue::StoreF32) {
    constexpr int kPerRow = WN / 4, kRowStep = 64 / kPerRow, kIters = (32 + kRowStep - 1) / kRowStep;
    const int c = (lane % kPerRow) * 4, n = col_base + c, row0 = lane / kPerRow;
    const bool active = n < p.N && lane < kPerRow * kRowStep, whole = n + 4 <= p.N;
    f32x4 b = {0.f, 0.f, 0.f, 0.f};
    if (p.bias && whole) {
      const uint2 bb = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(p.bias) + n);
      b[0] = __uint_as_float(bb.x << 16); b[1] = __uint_as_float(bb.x & 0xFFFF0000u);
      b[2] = __uint_as_float(bb.y << 16); b[3] = __uint_as_float(bb.y & 0xFFFF0000u);
    }
    const float* from = stage + row0 * kPitch + c;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      park(i);
      if (!active) continue;
      float* to = static_cast<float*>(p.C) + c_offset + (size_t)(row_base + i * 32 + row0) * p.ldc + n;
#pragma unroll
      for (int it = 0; it < kIters; ++it) {
        const int row = row0 + it * kRowStep, m = row_base + i * 32 + row;
        if (row >= 32 || m >= p.M) break;
        const f32x4 v = *reinterpret_cast<const f32x4*>(from + it * kRowStep * kPitch);
        if (whole) *reinterpret_cast<f32x4*>(to + (size_t)it * kRowStep * p.ldc) = v * p.alpha + b;
        else store_ragged(p, from + it * kRowStep * kPitch, 4, m, n, c_offset);   // straight from the parked row (a copy would live in scratch memory)
      }
    }
    return;
  }
  constexpr int kPerRow = WN / 8, kRowStep = 64 / kPerRow, kIters = (32 + kRowStep - 1) / kRowStep;
  const int c = (lane % kPerRow) * 8, n = col_base + c, row0 = lane / kPerRow;
  const bool active = n < p.N && lane < kPerRow * kRowStep, whole = n + 8 <= p.N;
  const int mode = p.epilogue;
  const bool plain = mode == (int)Epilogue::BiasAct;
  bf16_t* aux = plain ? static_cast<bf16_t*>(p.aux_out) : nullptr;
  const bf16_t* xsrc = plain ? static_cast<const bf16_t*>(p.residual) : static_cast<const bf16_t*>(p.mask);
  const int ldx = plain ? p.ldres : p.ldmask;
  const int last_row = p.M - 1;
  const bool scaled = p.alpha != 1.f;
  const float* from = stage + row0 * kPitch + c;
  auto request = [&](int i, u32x4 (&dst)[kIters]) {
    if (xsrc == nullptr || !active || !whole) return;
#pragma unroll
    for (int it = 0; it < kIters; ++it)  // from a clamped, always valid row
      dst[it] = *reinterpret_cast<const u32x4*>(xsrc + (size_t)min(row_base + i * 32 + row0 + it * kRowStep, last_row) * ldx + n);
  };
  // math(v, x, pre): v = alpha * acc on entry and the result on return; x = the per-element tensor's 8 values (only
  // with has_x); pre = what the auxiliary output stores (only worked out with has_aux).  Both flags are template
  // arguments of the variant so that a product without those tensors spends no instruction on them.
  // (always_inline: for large wave tiles the inliner otherwise leaves this body a function, and the accumulators,
  // passed by reference, then live in scratch memory through the whole tile loop)
  auto run = [&](auto has_x, auto has_aux, auto&& math) __attribute__((always_inline)) {
    constexpr bool kX = decltype(has_x)::value, kAux = decltype(has_aux)::value;
    u32x4 xs[2][kIters];
    if constexpr (kX) request(0, xs[0]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      park(i);
      if constexpr (kX) { if (i + 1 < TM) request(i + 1, xs[(i + 1) & 1]); }
      if (!active) continue;
      if (!whole) {  // ragged right edge: element by element
#pragma unroll 1
        for (int row = row0; row < 32 && row_base + i * 32 + row < p.M; row += kRowStep)
          store_ragged(p, stage + row * kPitch + c, 8, row_base + i * 32 + row, n, c_offset);
        continue;
      }
      const size_t first = (size_t)(row_base + i * 32 + row0);
      bf16_t* to = static_cast<bf16_t*>(p.C) + c_offset + first * p.ldc + n;
      bf16_t* to_aux = kAux ? aux + first * p.ldaux + n : nullptr;
#pragma unroll
      for (int it = 0; it < kIters; ++it) {
        const int row = row0 + it * kRowStep;
        if (row >= 32 || row_base + i * 32 + row >= p.M) break;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(from + it * kRowStep * kPitch);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(from + it * kRowStep * kPitch + 4);
        float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]}, x[8], pre[8];
        if (scaled) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= p.alpha;
        }
        if constexpr (kX) unpack_bf16x8(xs[i & 1][it], x);
        math(has_x, has_aux, v, x, pre);
        if constexpr (kAux) *reinterpret_cast<u32x4*>(to_aux + (size_t)it * kRowStep * p.ldaux) = pack_bf16x8(pre);
        *reinterpret_cast<u32x4*>(to + (size_t)it * kRowStep * p.ldc) = pack_bf16x8(v);
      }
    }
  };
  using Yes = std::true_type;
  using No = std::false_type;
  if (mode == (int)Epilogue::AffineBwdStore) {
    // (the columns are whole 16-byte pieces here: the host accepts the mode only for N % 8 == 0)
    const bf16_t* ysrc = static_cast<const bf16_t*>(p.affine_y);
    float sc[8];
    {
      u32x4 scw = {0u, 0u, 0u, 0u};
      if (active) scw = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(p.col_scale) + n);
      unpack_bf16x8(scw, sc);
    }
    float s_dzy[8], s_dz[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { s_dzy[e] = 0.f; s_dz[e] = 0.f; }
    // A lane's units (8 outputs each) in order: piece by piece, kIters rows per piece.  The two per-element chunks
    // of unit u + 2 are requested before unit u is worked out and stored: three sets of registers in rotation, and
    // waiting for a chunk never waits for a store issued after it.
    constexpr int kUnits = TM * kIters;
    auto unit_row = [&](int u) { return row_base + (u / kIters) * 32 + row0 + (u % kIters) * kRowStep; };
    // Optional: a second gradient that joins the product before the rounding (the shortcut's, where the product is a
    // unit's last input gradient) and a copy of dz itself (what that unit hands down its own shortcut).
    const bf16_t* rsrc = static_cast<const bf16_t*>(p.residual);
    bf16_t* dz_out = static_cast<bf16_t*>(p.aux_out);
    u32x4 ab[3], yb[3], rb[3];
    auto request2 = [&](int u, u32x4& a, u32x4& y, u32x4& r) {
      if (!active) return;
      const size_t row = (size_t)min(unit_row(u), last_row);   // a clamped, always valid row
      a = *reinterpret_cast<const u32x4*>(xsrc + row * ldx + n);
      y = *reinterpret_cast<const u32x4*>(ysrc + row * p.ldy + n);
      if (rsrc) r = *reinterpret_cast<const u32x4*>(rsrc + row * p.ldres + n);
    };
    request2(0, ab[0], yb[0], rb[0]);
    if constexpr (kUnits > 1) request2(1, ab[1], yb[1], rb[1]);
    static_for<kUnits>([&](auto u_c) {
      constexpr int u = decltype(u_c)::value, i = u / kIters, it = u % kIters;
      if constexpr (it == 0) park(i);
      if constexpr (u + 2 < kUnits) request2(u + 2, ab[(u + 2) % 3], yb[(u + 2) % 3], rb[(u + 2) % 3]);
      const int row = row0 + it * kRowStep;
      if (active && row < 32 && row_base + i * 32 + row < p.M) {
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(from + it * kRowStep * kPitch);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(from + it * kRowStep * kPitch + 4);
        float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]}, a[8], y[8], d[8], o[8];
        if (scaled) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= p.alpha;
        }
        if (rsrc) {
          float r[8];
          unpack_bf16x8(rb[u % 3], r);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += r[e];
        }
        unpack_bf16x8(pack_bf16x8(v), d);   // the gradient as a separate pass would have read it back from memory
        unpack_bf16x8(ab[u % 3], a);
        unpack_bf16x8(yb[u % 3], y);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (!(a[e] > 0.f)) d[e] = 0.f;
          s_dzy[e] += d[e] * y[e];
          s_dz[e] += d[e];
          o[e] = sc[e] * d[e];
        }
        const size_t m = (size_t)(row_base + i * 32 + row);
        if (dz_out) *reinterpret_cast<u32x4*>(dz_out + m * p.ldaux + n) = pack_bf16x8(d);   // exact: d is bfloat16 already
        *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(p.C) + c_offset + m * p.ldc + n) = pack_bf16x8(o);
      }
    });
    // Column sums: first over the lanes of this wave that share a column (their sums side by side in the wave's
    // staging rows, added in lane order), then over the WAVES_M waves that share it, in wave order.
    constexpr int kCols = 2 * WN;                       // [dz * y | dz] of the wave's WN columns
    constexpr int kPerLane = (kCols + 63) / 64;
    static_assert(kRowStep * kCols <= 32 * kPitch, "the lanes' column sums fit in the wave's staging rows");
    asm volatile("" ::: "memory");
    if (lane < kPerRow * kRowStep) {
      float* mine = stage + (lane / kPerRow) * kCols + c;
#pragma unroll
      for (int e = 0; e < 8; ++e) { mine[e] = s_dzy[e]; mine[WN + e] = s_dz[e]; }
    }
    asm volatile("" ::: "memory");
    float wave_sum[kPerLane];
#pragma unroll
    for (int u = 0; u < kPerLane; ++u) {
      const int col = lane + 64 * u;
      float t = 0.f;
      if (col < kCols) {
#pragma unroll
        for (int r = 0; r < kRowStep; ++r) t += stage[r * kCols + col];
      }
      wave_sum[u] = t;
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int u = 0; u < kPerLane; ++u)
      if (lane + 64 * u < kCols) stage[lane + 64 * u] = wave_sum[u];
    __syncthreads();
    if (wm == 0) {
#pragma unroll
      for (int u = 0; u < kPerLane; ++u) {
        const int col = lane + 64 * u;
        if (col >= kCols) continue;
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES_M; ++w) t += stage[w * (32 * kPitch) + col];   // wave wm + WAVES_M * wn: this column block's waves lie side by side
        const int which = col / WN, cn = col_base + col % WN;
        if (cn < p.N) p.col_partial[((size_t)tile_m * 2 + which) * p.N + cn] = t;
      }
    }
    return;
  }
  if (mode == (int)Epilogue::MaskStore) {
    run(Yes{}, No{}, [](auto, auto, float (&v)[8], const float (&x)[8], float (&)[8]) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = x[e] > 0.f ? v[e] : 0.f;
    });
    return;
  }
  if (mode == (int)Epilogue::ScaleStore) {
    run(Yes{}, No{}, [](auto, auto, float (&v)[8], const float (&x)[8], float (&)[8]) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] *= x[e];
    });
    return;
  }
  ColumnOperands cols;
  load_column_operands<WN>(p, col_base, lane, cols);
  float sc[8], bs[8];
  unpack_bf16x8(cols.sc, sc);
  unpack_bf16x8(cols.bs, bs);
  const bool aux_raw = p.aux_raw != 0;
  // v = v * s + b; pre = that (or the unscaled product); a residual joins before the activation
  auto affine = [&](auto has_x, auto has_aux, float (&v)[8], const float (&x)[8], float (&pre)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float t = v[e] * sc[e] + bs[e];
      if constexpr (decltype(has_aux)::value) pre[e] = aux_raw ? v[e] : t;
      if constexpr (decltype(has_x)::value) v[e] = t + x[e];
      else v[e] = t;
    }
  };
  // the four combinations of (residual, auxiliary output) of one activation
  auto variants = [&](auto&& math) __attribute__((always_inline)) {
    if (xsrc != nullptr) {
      if (aux != nullptr) run(Yes{}, Yes{}, math);
      else run(Yes{}, No{}, math);
    } else {
      if (aux != nullptr) run(No{}, Yes{}, math);
      else run(No{}, No{}, math);
    }
  };
  if (p.act == (int)Act::Relu) {
    variants([&](auto has_x, auto has_aux, float (&v)[8], const float (&x)[8], float (&pre)[8]) {
      affine(has_x, has_aux, v, x, pre);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
    });
  } else if (p.act == (int)Act::Gelu) {
    if (p.aux_act_grad && aux != nullptr) {  // the auxiliary output takes the activation's derivative
      auto both = [&](auto has_x, auto, float (&v)[8], const float (&x)[8], float (&pre)[8]) {
        affine(has_x, No{}, v, x, pre);
#pragma unroll
        for (int e = 0; e < 8; ++e) gelu_both_f(v[e], v[e], pre[e]);
      };
      if (xsrc != nullptr) run(Yes{}, Yes{}, both);
      else run(No{}, Yes{}, both);
    } else {
      variants([&](auto has_x, auto has_aux, float (&v)[8], const float (&x)[8], float (&pre)[8]) {
        affine(has_x, has_aux, v, x, pre);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
      });
    }
  } else {
    variants(affine);
  }
}

template <int BM, int BN, int STAGES, int WAVES_M, int WAVES_N, Layout LA, Layout LB, Gather GA, Gather GB>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_dma_kernel(GemmParams p) {
  constexpr int NW = WAVES_M * WAVES_N;
  static_assert(NW == 4 || NW == 8, "four or eight wavefronts per workgroup");
  static_assert(STAGES >= 2 && STAGES <= 8, "ring depth");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1 && WM % 32 == 0 && WN % 32 == 0, "wave tile is a multiple of 32x32");
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  constexpr int kLoadsPerTile = (BM + BN) / (8 * NW);  // direct-to-LDS instructions per wave per tile
  constexpr int kBatch = (TM + TN) <= 2 ? 4 : ((TM + TN) <= 4 ? 2 : 1);  // k-groups whose fragments are fetched together
  static_assert((size_t)NW * 32 * (WN + 4) * 4 <= (size_t)STAGES * kStageBytes, "epilogue staging fits in the tile ring");

  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int tile_m, tile_n;
  xcd_tile_grouped(p.slice_in_x ? blockIdx.y : blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  TileSource<BM, LA, GA, NW> src_a;
  TileSource<BN, LB, GB, NW> src_b;
  const int z = p.slice_in_x ? blockIdx.x : blockIdx.y;  // batch entry, or slice of the k range
  int t_first = 0, n_steps = (p.K + kTileK - 1) / kTileK;
  if (p.k_tiles_per_split > 0) {
    t_first = z * p.k_tiles_per_split;
    n_steps = min(n_steps, t_first + p.k_tiles_per_split);
  }
  src_a.init(static_cast<const bf16_t*>(p.A) + batch_offset_z(p.a_batch, z), p.lda, m0, p.M, wave, lane, t_first, p.conv);
  src_b.init(static_cast<const bf16_t*>(p.B) + batch_offset_z(p.b_batch, z), p.ldb, n0, p.N, wave, lane, t_first, p.conv);
  auto issue = [&](int t) {
    char* stage = lds + ((t - t_first) % STAGES) * kStageBytes;
    src_a.issue(t, p.K, stage, wave, p.lda, p.conv);
    src_b.issue(t, p.K, stage + BM * kRowBytes, wave, p.ldb, p.conv);
  };
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (t_first + s < n_steps) issue(t_first + s);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Bias gradient of a weight-gradient product: sum over k of A(row, k).  A KRow tile has 8 consecutive rows in
  // one 16-byte chunk, so a thread takes one chunk column and every kPhases-th k-row, keeps 8 partial sums and
  // the partial sums of the kPhases threads of a chunk are added up once, after the tile loop.
  constexpr int kChunks = BM / 8, kPhases = 64 * NW / kChunks;
  static_assert(kPhases >= 1 && kTileK % kPhases == 0 && (size_t)kPhases * BM * 4 <= (size_t)STAGES * kStageBytes, "row-sum partition");
  const bool want_row_sum = LA == Layout::KRow && p.a_row_sum != nullptr && tile_n == 0;
  float row_sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int sum_chunk = threadIdx.x % kChunks, sum_phase = threadIdx.x / kChunks;

  for (int t = t_first; t < n_steps; ++t) {
    // Tiles t+1 .. t+STAGES-2 may stay in flight if they were all issued; near the end wait for everything.
    if (t + STAGES - 2 < n_steps) wait_loads_and_barrier<(STAGES - 2) * kLoadsPerTile>();
    else wait_loads_and_barrier<0>();
    if (t + STAGES - 1 < n_steps) issue(t + STAGES - 1);
    const char* as = lds + ((t - t_first) % STAGES) * kStageBytes;
    const char* bs = as + BM * kRowBytes;
#pragma unroll
    for (int kb = 0; kb < 4; kb += kBatch) {
      u32x4 a[kBatch * TM], b[kBatch * TN];
#pragma unroll
      for (int g = 0; g < kBatch; ++g) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[g * TM + i] = read_fragment<BM, LA>(as, wm * WM + i * 32, kb + g, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[g * TN + j] = read_fragment<BN, LB>(bs, wn * WN + j * 32, kb + g, lane);
      }
      if constexpr (LA == Layout::KRow || LB == Layout::KRow) fragments_ready(a, b);
#pragma unroll
      for (int g = 0; g < kBatch; ++g)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b[g * TN + j]),   // operands exchanged:
                                                                __builtin_bit_cast(bf16x8, a[g * TM + i]), acc[i][j], 0, 0, 0);  // see store_wave_tile
      if constexpr (LA == Layout::RowK && LB == Layout::RowK) {
        // Keep the batch's LDS reads ahead of its MFMAs (the scheduler otherwise sinks each read to its use
        // and the wave eats one LDS latency per MFMA).
        __builtin_amdgcn_sched_group_barrier(0x100, kBatch * (TM + TN), 0);  // DS reads
        __builtin_amdgcn_sched_group_barrier(0x008, kBatch * TM * TN, 0);    // MFMA
      }
    }
    if constexpr (LA == Layout::KRow) {
      if (want_row_sum) {
#pragma unroll
        for (int j = 0; j < kTileK / kPhases; ++j) {
          const int k = sum_phase + j * kPhases;
          const int pc = (sum_chunk + krow_rot<BM>(k)) % kChunks;
          float f[8];
          unpack_bf16x8(*reinterpret_cast<const u32x4*>(as + k * (BM * 2) + pc * 16), f);
#pragma unroll
          for (int e = 0; e < 8; ++e) row_sum[e] += f[e];
        }
      }
    }
  }
  wait_loads_and_barrier<0>();  // every wave is done with the tile ring
  if constexpr (LA == Layout::KRow) {
    if (want_row_sum) {  // uniform over the workgroup
      float* part = reinterpret_cast<float*>(lds);
#pragma unroll
      for (int e = 0; e < 8; ++e) part[sum_phase * BM + sum_chunk * 8 + e] = row_sum[e];
      __syncthreads();
      if (threadIdx.x < BM) {
        float v = 0.f;
#pragma unroll
        for (int ph = 0; ph < kPhases; ++ph) v += part[ph * BM + threadIdx.x];
        if (m0 + (int)threadIdx.x < p.M) p.a_row_sum[m0 + threadIdx.x] = v;
      }
      __syncthreads();
    }
  }
  float* stage = reinterpret_cast<float*>(lds) + wave * (32 * (WN + 4));
  store_wave_tile<WM, WN, WAVES_M>(p, acc, stage, m0 + wm * WM, n0 + wn * WN, lane, batch_offset_z(p.c_batch, z), wm, tile_m);
}

// The same product with the tile loop written as a software pipeline.  In the kernel above a wave does one thing
// at a time (issue a tile's loads, read LDS, multiply) and a workgroup's waves do it together, so the vector-memory
// path, the LDS and the matrix cores of a CU take turns.  Here every k-group (16 of k) is a block of MFMAs on the
// fragments fetched during the block before, and between those MFMAs the wave issues the LDS reads of the next
// k-group's fragments and its share of a later tile's direct-to-LDS loads, one instruction at a time: the three
// pipes run side by side, and the loads of a tile are spread over several blocks instead of arriving at the
// memory path in one burst.  One barrier per tile, in front of the tile's last k-group: by then a wave has all of
// the tile in registers (so the buffer may be overwritten: tile t + STAGES goes there, its parts issued in the
// blocks that follow) and knows its own loads of tile t + 1 have landed (so everybody may read it: the last block
// fetches tile t + 1's first fragments).
//   STAGES >= 3: a tile's loads in as many parts as the tile has blocks; they have STAGES - 2 tiles' time to land
//   (the tile being multiplied plus STAGES - 2 tiles may be on their way).
//   STAGES = 2 (tiles too large for three): 2 parts, in the block after the barrier and the one after that, which
//   leaves them two blocks to land.
template <int BM, int BN, int STAGES, int WAVES_M, int WAVES_N, int KGB, Layout LA, Layout LB, Gather GA, Gather GB>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_pipe_kernel(GemmParams p) {
  constexpr int NW = WAVES_M * WAVES_N;
  static_assert(NW == 4 || NW == 8, "four or eight wavefronts per workgroup");
  static_assert(STAGES >= 2 && STAGES <= 5, "ring depth");
  static_assert(KGB == 1 || KGB == 2, "k-groups per block");
  constexpr int NB = 4 / KGB;                          // blocks per tile
  constexpr int PARTS = STAGES >= 3 ? NB : NB / 2;     // a tile's loads: in every block, or in the two after the barrier
  static_assert(PARTS >= 1, "a ring of two stages needs four blocks per tile");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1 && WM % 32 == 0 && WN % 32 == 0, "wave tile is a multiple of 32x32");
  constexpr int kMfma = KGB * TM * TN, kReads = KGB * (TM + TN);   // per block
  constexpr int kReadsPerSlot = (kReads + kMfma - 1) / kMfma;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  using SourceA = TileSource<BM, LA, GA, NW>;
  using SourceB = TileSource<BN, LB, GB, NW>;
  constexpr int kLoadsPerTile = SourceA::kInstr + SourceB::kInstr;
  static_assert((STAGES - 2) * kLoadsPerTile < 64, "vmcnt range");

  static_assert((size_t)NW * 32 * (WN + 4) * 4 <= (size_t)STAGES * kStageBytes, "epilogue staging fits in the tile ring");
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int tile_m, tile_n;
  xcd_tile_grouped(p.slice_in_x ? blockIdx.y : blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  SourceA src_a;
  SourceB src_b;
  const int z = p.slice_in_x ? blockIdx.x : blockIdx.y;  // batch entry, or slice of the k range
  int t_first = 0, n_steps = (p.K + kTileK - 1) / kTileK;
  if (p.k_tiles_per_split > 0) {
    t_first = z * p.k_tiles_per_split;
    n_steps = min(n_steps, t_first + p.k_tiles_per_split);
  }
  const int n = max(n_steps - t_first, 0);          // tiles of this workgroup, numbered from 0 below
  src_a.init(static_cast<const bf16_t*>(p.A) + batch_offset_z(p.a_batch, z), p.lda, m0, p.M, wave, lane, t_first, p.conv);
  src_b.init(static_cast<const bf16_t*>(p.B) + batch_offset_z(p.b_batch, z), p.ldb, n0, p.N, wave, lane, t_first, p.conv);
  auto stage_of = [&](int t) { return lds + (t % STAGES) * kStageBytes; };
  auto issue_part = [&](int t, int part) {           // tiles in increasing order, a tile's parts in increasing order
    if (t >= n) return;
    char* stage = stage_of(t);
    src_a.template issue<PARTS>(t_first + t, p.K, stage, wave, p.lda, p.conv, part);
    src_b.template issue<PARTS>(t_first + t, p.K, stage + BM * kRowBytes, wave, p.ldb, p.conv, part);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // bias gradient of a weight-gradient product (see the kernel above): the k-rows are fetched in a tile's first
  // block and added in its second
  constexpr int kChunks = BM / 8, kPhases = 64 * NW / kChunks, kSumReads = kTileK / kPhases;
  static_assert(kPhases >= 1 && kTileK % kPhases == 0 && (size_t)kPhases * BM * 4 <= (size_t)STAGES * kStageBytes, "row-sum partition");
  const bool want_row_sum = LA == Layout::KRow && p.a_row_sum != nullptr && tile_n == 0;
  float row_sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int sum_chunk = threadIdx.x % kChunks, sum_phase = threadIdx.x / kChunks;
  u32x4 sum_rows[kSumReads];

  auto pin = [] { __builtin_amdgcn_sched_barrier(0); };   // the instruction scheduler moves nothing across this point
  auto lds_done = [] { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); };

  // Two sets of fragment registers: a block multiplies one while the reads of the next block fill the other.
  // Within a set: the A fragments of the block's k-groups, then the B fragments.
  u32x4 fa[2][KGB * TM], fb[2][KGB * TN];
  auto keep = [&](int b) {
#pragma unroll
    for (int i = 0; i < KGB * TM; ++i) asm volatile("" : "+v"(fa[b][i]));
#pragma unroll
    for (int j = 0; j < KGB * TN; ++j) asm volatile("" : "+v"(fb[b][j]));
  };
  using ReaderA = FragmentReader<BM, LA, TM>;
  using ReaderB = FragmentReader<BN, LB, TN>;
  ReaderA reader_a;
  ReaderB reader_b;
  reader_a.init(wm * WM, lane);
  reader_b.init(wn * WN, lane);
  uint32_t at_a[ReaderA::kN], at_b[ReaderB::kN];       // the tile being multiplied
  uint32_t next_a[ReaderA::kN], next_b[ReaderB::kN];   // the tile after it (its first block is fetched during this tile's last)
  auto lds_address = [&](int t) { return (uint32_t)(uintptr_t)(lds_ptr_t)stage_of(t); };
  // read number R (0 .. kReads-1) of the block that starts at k-group KG0, from the tile at (a, b), into set `set`
  auto fetch = [&](auto set, auto kg0, auto r, const uint32_t (&a)[ReaderA::kN], const uint32_t (&b)[ReaderB::kN]) {
    constexpr int S = decltype(set)::value, KG0 = decltype(kg0)::value, R = decltype(r)::value;
    if constexpr (R < KGB * TM) fa[S][R] = ReaderA::template read<R % TM, KG0 + R / TM>(a);
    else if constexpr (R < kReads) fb[S][R - KGB * TM] = ReaderB::template read<(R - KGB * TM) % TN, KG0 + (R - KGB * TM) / TN>(b);
  };

  // ---- prologue: tiles 0 .. STAGES-2 whole, the first part of tile STAGES-1, then tile 0's first fragments
#pragma unroll
  for (int t = 0; t < STAGES - 1; ++t)
#pragma unroll
    for (int part = 0; part < PARTS; ++part) issue_part(t, part);
  issue_part(STAGES - 1, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  pin();
  __builtin_amdgcn_s_barrier();
  pin();
  if (n > 0) {
    reader_a.at(lds_address(0), next_a);
    reader_b.at(lds_address(0) + BM * kRowBytes, next_b);
    static_for<kReads>([&](auto r) { fetch(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, r, next_a, next_b); });
  }

  for (int t = 0; t < n; ++t) {
    const bool more = t + 1 < n;
    reader_a.at(lds_address(t), at_a);
    reader_b.at(lds_address(t) + BM * kRowBytes, at_b);
    const char* as = stage_of(t);
    static_for<NB>([&](auto blk_c) {
      constexpr int blk = decltype(blk_c)::value;
      constexpr int cur = blk & 1, nxt = cur ^ 1;
      constexpr bool last = blk == NB - 1;
      // ---- the fragments of this block are in registers
      lds_done();
      keep(cur);
      if constexpr (LA == Layout::KRow) {
        if (blk == 1 && want_row_sum) {
#pragma unroll
          for (int r = 0; r < kSumReads; ++r) {
            asm volatile("" : "+v"(sum_rows[r]));
            float f[8];
            unpack_bf16x8(sum_rows[r], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) row_sum[e] += f[e];
          }
        }
      }
      if constexpr (last) {
        // All of tile t is in registers; this wave's loads of tile t + 1 have landed (the STAGES - 2 tiles after it may
        // stay in flight when all of them have been issued).
        if (STAGES >= 3 && t + STAGES - 1 < n) __builtin_amdgcn_s_waitcnt(waitcnt_imm((STAGES - 2) * kLoadsPerTile, 15));
        else __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));
        pin();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        reader_a.at(lds_address(t + 1), next_a);
        reader_b.at(lds_address(t + 1) + BM * kRowBytes, next_b);
      }
      pin();
      // ---- MFMAs of this block; between them the next block's fragment reads and one part of a later tile's loads
      constexpr int kg_next = last ? 0 : (blk + 1) * KGB;
      const bool fetching = !last || more;
      const int load_tile = last ? t + STAGES : t + STAGES - 1;   // part 0 right after the barrier, the others in the next tile's blocks
      constexpr int load_part = last ? 0 : blk + 1;
      static_for<kMfma>([&](auto idx_c) {
        constexpr int idx = decltype(idx_c)::value;
        constexpr int g = idx / (TM * TN), i = (idx / TN) % TM, j = idx % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[cur][g * TN + j]),   // operands exchanged:
                                                            __builtin_bit_cast(bf16x8, fa[cur][g * TM + i]), acc[i][j], 0, 0, 0);  // see store_wave_tile
        if (fetching) {
          static_for<kReadsPerSlot>([&](auto q) {
            constexpr int r = idx * kReadsPerSlot + decltype(q)::value;
            if constexpr (last) fetch(std::integral_constant<int, nxt>{}, std::integral_constant<int, kg_next>{}, std::integral_constant<int, r>{}, next_a, next_b);
            else fetch(std::integral_constant<int, nxt>{}, std::integral_constant<int, kg_next>{}, std::integral_constant<int, r>{}, at_a, at_b);
          });
        }
        if constexpr (idx == 0 && load_part < PARTS) issue_part(load_tile, load_part);
        pin();
      });
      if constexpr (LA == Layout::KRow) {
        if (blk == 0 && want_row_sum) {
#pragma unroll
          for (int r = 0; r < kSumReads; ++r) {
            const int k = sum_phase + r * kPhases;
            const int pc = (sum_chunk + krow_rot<BM>(k)) % kChunks;
            sum_rows[r] = lds_read_b128_asm(as + k * (BM * 2) + pc * 16);
          }
          pin();
        }
      }
    });
  }
  lds_done();
  // Every wave is past the last tile's barrier, which it reached with the whole tile in registers: the ring is dead.
  __syncthreads();
  if constexpr (LA == Layout::KRow) {
    if (want_row_sum) {  // uniform over the workgroup
      float* part = reinterpret_cast<float*>(lds);
#pragma unroll
      for (int e = 0; e < 8; ++e) part[sum_phase * BM + sum_chunk * 8 + e] = row_sum[e];
      __syncthreads();
      if (threadIdx.x < BM) {
        float v = 0.f;
#pragma unroll
        for (int ph = 0; ph < kPhases; ++ph) v += part[ph * BM + threadIdx.x];
        if (m0 + (int)threadIdx.x < p.M) p.a_row_sum[m0 + threadIdx.x] = v;
      }
      __syncthreads();
    }
  }
  float* stage = reinterpret_cast<float*>(lds) + wave * (32 * (WN + 4));
  store_wave_tile<WM, WN, WAVES_M>(p, acc, stage, m0 + wm * WM, n0 + wn * WN, lane, batch_offset_z(p.c_batch, z), wm, tile_m);
}

// Small products (at most a few workgroups per CU) are a chain of latencies, not a throughput problem, and the
// one throughput that does bound them is a CU's vector-memory path of about 57 bytes per clock.  So: tiles small
// enough that every CU gets one (32 x 32 or 64 x 64), and no barrier in the tile loop at all: each of the four
// waves owns a contiguous quarter of the k range with a tile ring of its own in LDS, waits only on its own
// loads, and drifts freely against the others, which overlaps one wave's loads with another's LDS reads and
// MFMAs.  The four partial tiles are summed through LDS at the end, each wave finishing a quarter of the rows.
template <int VM>
__device__ __forceinline__ void wait_own_loads() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(VM, 15));
  asm volatile("" ::: "memory");
}

// LDS of one small-product workgroup whose waves keep SW tiles each: the four rings, or the four parked
// partial tiles where those need more.
constexpr size_t small_product_lds(int bm, int bn, int sw) {
  const size_t rings = (size_t)4 * sw * (bm + bn) * kRowBytes, parked = (size_t)4 * bm * (bn + 4) * 4;
  return (rings > parked ? rings : parked + 1023) / 1024 * 1024;
}

template <int BM, int BN, int SW, Layout LA, Layout LB>
__device__ __forceinline__ void small_product(const GemmParams& p, int block, int z, char* lds) {
  constexpr int NW = 4, TM = BM / 32, TN = BN / 32;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;  // SW of them per wave
  constexpr int kLoads = (BM + BN) / 8;        // direct-to-LDS instructions per tile (one wave loads a whole tile)
  constexpr int kPitch = BN + 4;               // floats per parked row; column BN carries the row sum of A
  constexpr int kRows = BM / NW;               // rows each wave finishes
  static_assert((BM == 32 || BM == 64) && (BN == 32 || BN == 64), "small tiles");
  static_assert(SW >= 1 && SW * kLoads < 64, "vmcnt range");

  const int tile = xcd_tile(block, p.tiles_m * p.tiles_n);
  const int tile_m = tile % p.tiles_m, tile_n = tile / p.tiles_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* ring = lds + wave * (SW * kStageBytes);

  int t_first = 0, t_end = (p.K + kTileK - 1) / kTileK;
  if (p.k_tiles_per_split > 0) {
    t_first = z * p.k_tiles_per_split;
    t_end = min(t_end, t_first + p.k_tiles_per_split);
  }
  const int per_wave = (max(t_end - t_first, 0) + NW - 1) / NW;
  const int my_first = t_first + wave * per_wave;
  const int n = max(min(t_end, my_first + per_wave) - my_first, 0);  // tiles of this wave

  TileSource<BM, LA, Gather::None, 1> src_a;
  TileSource<BN, LB, Gather::None, 1> src_b;
  src_a.init(static_cast<const bf16_t*>(p.A) + batch_offset_z(p.a_batch, z), p.lda, m0, p.M, 0, lane, my_first, p.conv);
  src_b.init(static_cast<const bf16_t*>(p.B) + batch_offset_z(p.b_batch, z), p.ldb, n0, p.N, 0, lane, my_first, p.conv);
  auto issue = [&](int i) {  // i-th tile of this wave, into its ring slot i % SW
    char* stage = ring + (i % SW) * kStageBytes;
    src_a.issue(my_first + i, p.K, stage, 0, p.lda, p.conv);
    src_b.issue(my_first + i, p.K, stage + BM * kRowBytes, 0, p.ldb, p.conv);
  };
#pragma unroll
  for (int s = 0; s < SW; ++s)
    if (s < n) issue(s);

  ColumnOperands cols;  // what the epilogue reads from global memory: requested now, used after the tile loop
  u32x4 xpre[2];
  static_assert(kRows <= 2 * (64 / (BN / 8)), "two epilogue rows per lane at most");
  load_column_operands<BN>(p, n0, lane, cols);
  load_row_operands<BN>(p, m0 + kRows * wave, n0, lane, xpre);

  f32x16 acc[TM][TN], acc_sum[TM];
#pragma unroll
  for (int x = 0; x < TM; ++x) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      acc_sum[x][r] = 0.f;
#pragma unroll
      for (int y = 0; y < TN; ++y) acc[x][y][r] = 0.f;
    }
  }
  // bias gradient of a weight-gradient product: row sums of A, as one more MFMA against a fragment of ones
  const bool want_row_sum = p.a_row_sum != nullptr && tile_n == 0;
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};

  for (int i = 0; i < n; ++i) {
    // tile i has landed once only the tiles issued after it are still in flight
    const int younger = min(SW - 1, n - 1 - i);
    if (younger == SW - 1) wait_own_loads<(SW - 1) * kLoads>();
    else if (SW > 2 && younger == 2) wait_own_loads<2 * kLoads>();
    else if (SW > 2 && younger == 1) wait_own_loads<1 * kLoads>();
    else wait_own_loads<0>();
    const char* as = ring + (i % SW) * kStageBytes;
    const char* bs = as + BM * kRowBytes;
    u32x4 a[4 * TM], b[4 * TN];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int x = 0; x < TM; ++x) a[g * TM + x] = read_fragment<BM, LA>(as, x * 32, g, lane);
#pragma unroll
      for (int y = 0; y < TN; ++y) b[g * TN + y] = read_fragment<BN, LB>(bs, y * 32, g, lane);
    }
    fragments_ready(a, b);  // the slot is free again
    if (i + SW < n) issue(i + SW);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y)
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[g * TM + x]), __builtin_bit_cast(bf16x8, b[g * TN + y]), acc[x][y], 0, 0, 0);
      if (want_row_sum) {
#pragma unroll
        for (int x = 0; x < TM; ++x)
          acc_sum[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[g * TM + x]), __builtin_bit_cast(bf16x8, ones), acc_sum[x], 0, 0, 0);
      }
    }
  }
  wait_loads_and_barrier<0>();  // every wave is done with its ring: park the partial tiles there

  float* red = reinterpret_cast<float*>(lds);
  float* mine = red + wave * (BM * kPitch);
#pragma unroll
  for (int x = 0; x < TM; ++x) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 32 * x + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
#pragma unroll
      for (int y = 0; y < TN; ++y) mine[row * kPitch + 32 * y + (lane & 31)] = acc[x][y][r];
      if (want_row_sum && (lane & 31) == 0) mine[row * kPitch + BN] = acc_sum[x][r];
    }
  }
  __syncthreads();
  // wave w finishes rows kRows * w ..: the row loops add up the four partials
  const int row_base = kRows * wave;
  if (want_row_sum && lane < kRows) {
    const float* at = red + (row_base + lane) * kPitch + BN;
    const float v = at[0] + at[BM * kPitch] + at[2 * BM * kPitch] + at[3 * BM * kPitch];
    if (m0 + row_base + lane < p.M) p.a_row_sum[m0 + row_base + lane] = v;
  }
  const float* stage = red + row_base * kPitch;
  if (p.epilogue == (int)Epilogue::StoreF32) store_rows_f32<BN, NW>(p, stage, m0 + row_base, n0, lane, batch_offset_z(p.c_batch, z), kRows, BM * kPitch);
  else store_rows_bf16<BN, NW>(p, stage, m0 + row_base, n0, lane, batch_offset_z(p.c_batch, z), kRows, BM * kPitch, &cols, xpre);
}

// Ring depth per wave: alone on its CU a workgroup's rings fill 128 KiB; the workgroups of a pair launch take
// half, so that one of each product fits on a CU and their fixed latencies overlap.
constexpr int small_ring_depth(int bm, int bn, bool paired) { return (int)((paired ? 64 : 128) * 1024 / (4 * (bm + bn) * kRowBytes)); }

template <int BM, int BN, Layout LA, Layout LB>
__global__ __launch_bounds__(256) void gemm_bf16_small_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  small_product<BM, BN, small_ring_depth(BM, BN, false), LA, LB>(p, blockIdx.x, blockIdx.y /* batch entry, or slice of the k range */, lds);
}

// Two independent small products in one launch (the input gradient and the weight gradient of a dense layer,
// which both start from the same output gradient): the first product's tiles take the lower block indices.
template <int BM1, int BN1, Layout LA1, Layout LB1, int BM2, int BN2, Layout LA2, Layout LB2>
__global__ __launch_bounds__(256) void gemm_bf16_small_pair_kernel(GemmParams p1, GemmParams p2) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int n1 = p1.tiles_m * p1.tiles_n;
  if ((int)blockIdx.x < n1) small_product<BM1, BN1, small_ring_depth(BM1, BN1, true), LA1, LB1>(p1, blockIdx.x, 0, lds);
  else small_product<BM2, BN2, small_ring_depth(BM2, BN2, true), LA2, LB2>(p2, blockIdx.x - n1, 0, lds);
}
template <int BM1, int BN1, int BM2, int BN2>
constexpr size_t small_pair_lds() {
  const size_t a = small_product_lds(BM1, BN1, small_ring_depth(BM1, BN1, true)), b = small_product_lds(BM2, BN2, small_ring_depth(BM2, BN2, true));
  return a > b ? a : b;
}


// Which products go to the small-product kernel, and with which tile.  Its workgroups take most of a CU's LDS,
// so it is for products with at most one tile per CU; with more 64 x 64 tiles than that, two or three
// workgroups of the ring kernel per CU do better.
inline long tile_count(const GemmProblem& q, int tm, int tn) { return (long)((q.M + tm - 1) / tm) * ((q.N + tn - 1) / tn) * q.batch * q.k_splits; }
inline bool small_product_fits(const GemmProblem& q) {
  if (q.a_gather != Gather::None || q.b_gather != Gather::None) return false;
  if (q.N <= 64 && q.M > 64) return tile_count(q, 256, 64) < 256;
  if (q.M <= 64 && q.N > 64) return tile_count(q, 64, 256) < 256;
  return tile_count(q, 128, 128) < 192 && tile_count(q, 64, 64) <= 256;
}
// 32 x 32 tiles only while they still make a single round over the CUs.
inline bool small_product_tile64(const GemmProblem& q) { return tile_count(q, 64, 64) >= 192 || tile_count(q, 32, 32) > 256; }

template <int BM, int BN, Layout LA, Layout LB>
hipError_t launch_small(const GemmProblem& q, hipStream_t stream) {
  GemmParams p = make_params(q, BM, BN);
  int grid_y = q.batch;
  if (q.k_splits > 1) {
    const int tiles = (q.K + kTileK - 1) / kTileK;
    p.k_tiles_per_split = (tiles + q.k_splits - 1) / q.k_splits;
    p.c_batch.outer = (long long)q.M * q.ldc; p.c_batch.inner = 0; p.c_batch.inner_count = 1;
    grid_y = q.k_splits;
  }
  constexpr size_t lds_bytes = small_product_lds(BM, BN, small_ring_depth(BM, BN, false));
  auto kernel = gemm_bf16_small_kernel<BM, BN, LA, LB>;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kernel), lds_bytes); e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(p.tiles_m * p.tiles_n, grid_y), dim3(256), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int BM, int BN, int STAGES, int WAVES_M, int WAVES_N, Layout LA, Layout LB, Gather GA, Gather GB>
hipError_t launch_tile(const GemmProblem& q, hipStream_t stream) {
  GemmParams p = make_params(q, BM, BN);
  int grid_y = q.batch;
  if (q.k_splits > 1) {
    const int tiles = (q.K + kTileK - 1) / kTileK;
    p.k_tiles_per_split = (tiles + q.k_splits - 1) / q.k_splits;
    p.c_batch.outer = (long long)q.M * q.ldc; p.c_batch.inner = 0; p.c_batch.inner_count = 1;
    grid_y = q.k_splits;
  }
  constexpr size_t lds_bytes = (size_t)STAGES * (BM + BN) * kRowBytes;
  static_assert(lds_bytes <= 160 * 1024, "LDS of one CU");
  auto kernel = gemm_bf16_dma_kernel<BM, BN, STAGES, WAVES_M, WAVES_N, LA, LB, GA, GB>;
  if (lds_bytes > 64 * 1024)
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kernel), lds_bytes); e != hipSuccess) return e;
  p.slice_in_x = q.k_splits > 1 && q.k_splits % 8 == 0 && p.tiles_m * p.tiles_n <= 65535;
  const dim3 grid = p.slice_in_x ? dim3(grid_y, p.tiles_m * p.tiles_n) : dim3(p.tiles_m * p.tiles_n, grid_y);
  hipLaunchKernelGGL(kernel, grid, dim3(64 * WAVES_M * WAVES_N), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int BM, int BN, int STAGES, int WAVES_M, int WAVES_N, int KGB, Layout LA, Layout LB, Gather GA, Gather GB>
hipError_t launch_tile_pipe(const GemmProblem& q, hipStream_t stream) {
  GemmParams p = make_params(q, BM, BN);
  int grid_y = q.batch;
  if (q.k_splits > 1) {
    const int tiles = (q.K + kTileK - 1) / kTileK;
    p.k_tiles_per_split = (tiles + q.k_splits - 1) / q.k_splits;
    p.c_batch.outer = (long long)q.M * q.ldc; p.c_batch.inner = 0; p.c_batch.inner_count = 1;
    grid_y = q.k_splits;
  }
  constexpr size_t lds_bytes = (size_t)STAGES * (BM + BN) * kRowBytes;
  static_assert(lds_bytes <= 160 * 1024, "LDS of one CU");
  auto kernel = gemm_bf16_pipe_kernel<BM, BN, STAGES, WAVES_M, WAVES_N, KGB, LA, LB, GA, GB>;
  if (lds_bytes > 64 * 1024)
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kernel), lds_bytes); e != hipSuccess) return e;
  p.slice_in_x = q.k_splits > 1 && q.k_splits % 8 == 0 && p.tiles_m * p.tiles_n <= 65535;
  const dim3 grid = p.slice_in_x ? dim3(grid_y, p.tiles_m * p.tiles_n) : dim3(p.tiles_m * p.tiles_n, grid_y);
  hipLaunchKernelGGL(kernel, grid, dim3(64 * WAVES_M * WAVES_N), lds_bytes, stream, p);
  return hipGetLastError();
}

// Tile choice.  A 256 x 256 tile reads half as many operand bytes per flop from L2 as a 128 x 128 one, which is
// what large products need.  A
// dimension of 64 or less (a 64-channel convolution) gets a 64-wide tile so that no matrix-core work is spent
// on rows that do not exist.  Products with too few tiles for that go to the small-product kernel (plain
// operands) or to 64 x 64 tiles with a deeper ring (gathered operands): they are bound by latency.
template <Layout LA, Layout LB, Gather GA = Gather::None, Gather GB = Gather::None>
hipError_t launch_layouts(const GemmProblem& q, hipStream_t stream) {
  auto tiles = [&](int tm, int tn) { return tile_count(q, tm, tn); };
  if constexpr (GA == Gather::None && GB == Gather::None) {
    if (small_product_fits(q) && q.epilogue != Epilogue::AffineBwdStore) {   // (the small kernel's epilogue has no column sums)
      if (small_product_tile64(q)) return launch_small<64, 64, LA, LB>(q, stream);
      return launch_small<32, 32, LA, LB>(q, stream);
    }
  }
  if (q.N <= 64 && q.M > 64) {
    // 128 x 64 with three stages leaves room for two workgroups per CU, which beat one of 256 x 64 by 10-30 %
    if (tiles(128, 64) >= 512) return launch_tile<128, 64, 3, 4, 1, LA, LB, GA, GB>(q, stream);
    return launch_tile<64, 64, 4, 2, 2, LA, LB, GA, GB>(q, stream);
  }
  if (q.M <= 64 && q.N > 64) {
    if (tiles(64, 256) >= 256) return launch_tile<64, 256, 3, 1, 4, LA, LB, GA, GB>(q, stream);
    return launch_tile<64, 64, 4, 2, 2, LA, LB, GA, GB>(q, stream);
  }
  // 256 x 256 when its tiles make whole rounds over the 256 CUs: one round that covers most of the chip beats
  // one and a half rounds of 128 x 128 tiles, and so do many rounds; a round and a bit does not.
  // A 256 x 192 tile when that makes ONE round with (nearly) every CU busy: 3072 or 2304 columns against 4096
  // rows give 256 or 192 such tiles where 256 x 256 gives 192 or 144.
  const long t192 = tiles(256, 192);
  if (q.M >= 256 && t192 >= 176 && t192 <= 256 && (long)((q.N + 191) / 192) * 192 * 20 <= (long)q.N * 21)
    return launch_tile<256, 192, 2, 4, 2, LA, LB, GA, GB>(q, stream);
  const long t256 = tiles(256, 256);
  // (a k range of one or two tiles has nothing to reuse: such products are bound by memory and run better as two
  // 128 x 128 workgroups per CU)
  if (q.M >= 256 && q.N >= 256 && q.K > 128 && t256 >= 176 && (t256 <= 256 || t256 >= 448)) return launch_tile_pipe<256, 256, 2, 2, 4, 1, LA, LB, GA, GB>(q, stream);
  // 128 x 128: two workgroups per CU hide each other's barriers when there are tiles for that; a workgroup
  // alone on its CU keeps three tiles in flight instead (a four-stage ring; a fifth stage measured slower).
  if (tiles(128, 128) > 256) return launch_tile<128, 128, 2, 2, 2, LA, LB, GA, GB>(q, stream);
  // Weight gradients of the encoder's dense layers (K = tokens): 108-144 tiles of 128 x 128.  Alone on the chip that
  // is level with 576 tiles of 64 x 64, but these products run beside the input-gradient chain of the other stream,
  // and there the big tiles do the same work in half the CU time and leave the other CUs to that chain (+5 % on the
  // encoder step; the four-wave kernels with two or three stages gave +1 and +3 %).
  // The k-slices of a convolution's weight gradient (gathered patches along k) likewise: +0.7 % on the bottleneck CNN.
  if constexpr (LA == Layout::KRow && LB == Layout::KRow) {
    if (tiles(128, 128) >= 96 && q.M >= 128 && q.N >= 128 && q.K >= 2048) return launch_tile_pipe<128, 128, 4, 2, 4, 2, LA, LB, GA, GB>(q, stream);
  }
  if (tiles(128, 128) >= 192) {
    // one round of lone workgroups: convolutions (gathered operands) did 2-5 % better as two 128 x 64 workgroups per
    // CU; plain products were level, and 128 x 128 leaves LDS for a weight-gradient workgroup of the second stream
    if constexpr (GA != Gather::None || GB != Gather::None) return launch_tile<128, 64, 3, 4, 1, LA, LB, GA, GB>(q, stream);
    else if (q.share_cu) return launch_tile<128, 128, 2, 2, 2, LA, LB, GA, GB>(q, stream);   // 64 KB of LDS instead of 128
    else return launch_tile_pipe<128, 128, 4, 2, 4, 2, LA, LB, GA, GB>(q, stream);   // eight waves: a lone workgroup needs two per SIMD to hide its own latencies
  }
  // 64 x 64: the ring depth that lets every tile be resident at once (two or three workgroups per CU).
  if (tiles(64, 64) > 512) return launch_tile<64, 64, 3, 2, 2, LA, LB, GA, GB>(q, stream);
  return launch_tile<64, 64, 4, 2, 2, LA, LB, GA, GB>(q, stream);
}

}  // namespace gemm_dma_detail
}  // namespace spb
