// One operand tile on its way global memory -> registers -> LDS -> matrix-core fragment, with the fused
// prologues (plain, transposed, element-aligned, img2col gather).
#pragma once

#include "config.hpp"

namespace hidet {

// ---------------------------------------------------------------------------------------------
// One operand (A or B) of one workgroup: global source + LDS tile.
//   ROWS   extent of the tile along M (for A) or N (for B)
//   LAYOUT L_KC: element (r, k) at src[r*ld + k];  L_MC: element (k, r) at src[k*ld + r]
// LDS layout, 16-bit types: same orientation as the source, chunk-swizzled (see swz_*).
// LDS layout, fp32: always [k][r] (each lane reads a single float per MFMA, consecutive lanes
// read consecutive r), so a KC source is transposed on its way into LDS.
// ---------------------------------------------------------------------------------------------
template <typename T, int ROWS, int BK, int LAYOUT, int MODE, int NT, int MI>
struct Operand {
  static constexpr bool IS_F32 = sizeof(T) == 4;
  static constexpr int VEC = 16 / (int)sizeof(T);
  static constexpr int CPR = (LAYOUT == L_KC) ? BK / VEC : ROWS / VEC;  // chunks per stored row
  static constexpr int SROWS = (LAYOUT == L_KC) ? ROWS : BK;             // stored rows
  static constexpr int NL = ROWS * BK / VEC / NT;
  static constexpr int KGROUPS = 64 / MI;
  using LoadMap = typename std::conditional<(IS_F32 && LAYOUT == L_KC), LoadMapColMajor<SROWS, CPR, NT>,
                                            LoadMapRowMajor<SROWS, CPR, NT>>::type;
  using Frag = typename FragT<T>::type;

  const T* src;      // origin of this workgroup's panel: row r0 (KC) or column r0 (MC), k = 0
  long long ld;
  int rows_left;     // valid extent along ROWS from the panel origin (may exceed ROWS, may be <= 0)
  int K;             // extent of this workgroup's K range
  int kofs;          // global k index where that range starts (needed by the img2col gather)
  int r0;            // global row/column of the panel origin (needed by the img2col gather)
  long long span;    // elements from `src` to the end of what the operand spans, (rows - 1) * ld + cols of one batch
                     // entry: a 16-byte access at offset o from `src` stays inside the operand iff o + VEC <= span

  // ---- global -> registers ------------------------------------------------------------------
  // Element mode, a chunk of a partial K tile: rows are not 16-byte aligned (odd leading dimension, offset
  // pointer).  A chunk that lies entirely inside the matrix is still fetched with one 16-byte load -- the address is
  // only element aligned, which global loads accept on this target -- and only chunks that straddle an edge fall
  // back to one load per element, each issued unconditionally from a clamped (always valid) address with the
  // predicate applied to the value, so that they are in flight together instead of waiting behind branches.
  __device__ __forceinline__ u32x4 gather(int sr, int sc, int k0) const {
    T tmp[VEC];
    {
      long long base;
      int valid;  // elements of the chunk inside the matrix
      bool whole;  // the 16 bytes of the chunk may be read at once
      if constexpr (LAYOUT == L_KC) {
        base = (long long)sr * ld + (k0 + sc);
        valid = sr < rows_left ? K - (k0 + sc) : 0;
        // a chunk that sticks out along K is read whole and masked below, unless it would leave the operand
        whole = valid >= VEC || (valid > 0 && base + VEC <= span);
      } else {
        base = (long long)(k0 + sr) * ld + sc;
        valid = k0 + sr < K ? rows_left - sc : 0;
        // a chunk that sticks out along M/N may be read whole (see init) unless it would leave the operand
        whole = valid >= VEC || (valid > 0 && base + VEC <= span);
      }
      if (valid <= 0) return u32x4{0u, 0u, 0u, 0u};
      if (whole) {
        u32x4 v = reinterpret_cast<const Unaligned*>(src + base)->v;
        if constexpr (LAYOUT == L_KC) {
          // along K what lies beyond the matrix must contribute exact zeros
          if (valid < VEC) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if constexpr (IS_F32)
                v[i] = valid > i ? v[i] : 0u;
              else
                v[i] &= valid >= 2 * i + 2 ? 0xffffffffu : (valid == 2 * i + 1 ? 0x0000ffffu : 0u);
            }
          }
        }
        return v;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const bool ok = e < valid;
        const T v = src[ok ? base + e : 0];
        tmp[e] = ok ? v : (T)0.0f;
      }
    }
    return __builtin_bit_cast(u32x4, tmp);
  }

  // Vector mode (LD_VEC): the host guarantees 16-byte aligned rows and that no chunk straddles the
  // edge of the matrix (K, resp. the M/N extent, is a multiple of the chunk length).  Chunks that lie
  // outside the matrix along M/N are redirected to the last valid row / chunk: they only feed output
  // rows or columns that are never stored, so any finite or non-finite value is harmless there.
  // Along K a chunk outside the matrix must read as zero; that can only happen in the last K tile.
  int off[NL];  // element offset of each chunk from `src` at k = 0 (vector mode only)
  // Element mode: the same idea at element alignment.  eoff = offset of the chunk at k = 0, nv = how many
  // of its VEC elements lie inside the matrix along M/N (a property of the chunk, not of the K tile).
  // Chunks entirely outside are redirected to a chunk inside (nv = VEC; they feed outputs that are never
  // stored).  A chunk that straddles the M/N edge is still read whole: the bytes past the edge are the
  // padding of the row or the beginning of the next row -- valid memory, and values that only reach
  // outputs that are never stored.  The exception is the last row of the operand, where "past the edge"
  // may be past the allocation: nv = -(valid elements) marks such chunks, and the one row concerned is
  // fetched element by element (so is everything in a matrix narrower than one chunk, 0 <= nv < VEC).
  static constexpr int NE = (MODE == LD_ELEM) ? NL : 1;
  long long eoff[NE];
  int nv[NE];
  struct __attribute__((packed, aligned(sizeof(T)))) Unaligned {
    u32x4 v;
  };
  // ---- img2col mode --------------------------------------------------------------------------------------
  // Stored row sr = k index (ic, kh, kw); a chunk = VEC consecutive output positions of one output row.  The load
  // map gives a thread the same chunk column in every row it loads, so what depends on the positions is one set
  // of values per thread, prepared by init(): the offset of the input pixel (image, oh*sh - ph, ow*sw - pw) of
  // channel 0 that element 0 of the chunk reads at (kh, kw) = (0, 0) (may be negative), that pixel's row and
  // column, and how many of the chunk's positions are real (ow < OW and inside the matrix).
  int pofs, ih0, iw0, pcnt;
  // A chunk is fetched in two phases so that the loads of all of a thread's chunks -- and the matrix-core work of
  // the current tile -- overlap their latency: request_window() forms the address and issues the load(s),
  // finish_window(), called when the tile is written to LDS, applies what depends on the loaded value.
  static constexpr bool GATHER = MODE == LD_IM2COL || MODE == LD_IM2COL_TAP;
  static constexpr int NP = GATHER ? NL : 1;
  u32x4 win2[NP];  // stride 2: the second half of the window
  u32x4 wmask[NP]; // the 16-byte mask that keeps elements [lo, hi)
  int wstart[NP];  // element offset of the window
  int winfo[NP];   // lo * (VEC + 1) + hi: elements [lo, hi) are kept; bit 8: the window leaves the tensor
  int wsw;         // 2: windows are 2 * VEC elements of which the even ones are used; else 1
  // Tap-major K order (LD_IM2COL_TAP): a K tile lies within one filter tap, so everything that depends on the tap
  // and on the thread's output positions -- the kept range [lo, hi), its mask, the spatial part of the window's
  // offset -- is the same for all of the thread's chunks of the tile and is worked out once per tile; a chunk then
  // costs one multiply-add for its channel, a bounds test and the load.
  u32x4 tmask;     // mask of the current tile
  int tinfo;       // lo * (VEC + 1) + hi of the current tile
  unsigned tedge;  // bit q: chunk q's window leaves the tensor (first or last pixels), fetched element-wise at the store
  // LDS table of 16-byte masks: entry lo * (VEC + 1) + hi keeps elements [lo, hi) of a chunk
  const unsigned char* masks;
  static constexpr int MASK_ENTRIES = (VEC + 1) * (VEC + 1);
  __device__ __forceinline__ void fill_masks(int tid, unsigned char* table) {
    if (tid < MASK_ENTRIES) {
      const int lo = tid / (VEC + 1), hi = tid % (VEC + 1);
      u32x4 m;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (IS_F32) {
          m[i] = (i >= lo && i < hi) ? 0xffffffffu : 0u;
        } else {
          m[i] = ((2 * i >= lo && 2 * i < hi) ? 0x0000ffffu : 0u) | ((2 * i + 1 >= lo && 2 * i + 1 < hi) ? 0xffff0000u : 0u);
        }
      }
      *reinterpret_cast<u32x4*>(table + tid * 16) = m;
    }
    masks = table;
  }

  __device__ __forceinline__ u32x4 request_window(int q, int sr, int k0, const ConvGeom& g) {
    const int kk = k0 + sr;
    const int k = kofs + kk;
    const int ic = g.d_khw.div(k), rem = k - ic * (g.KH * g.KW);
    const int kh = g.d_kw.div(rem), kw = rem - kh * g.KW;
    const int ih = ih0 + kh, iwf = iw0 + kw;  // input row, input column of element 0
    const bool row_ok = kk < K && (unsigned)ih < (unsigned)g.H;
    // (offsets of rows beyond K, which are masked, may wrap: unsigned arithmetic)
    const int start = (int)((unsigned)pofs + ((unsigned)ic * (unsigned)g.H + (unsigned)kh) * (unsigned)g.W + (unsigned)kw);
    if (g.sw <= 2 && g.numel_x >= 2 * VEC) {  // (a tensor smaller than the window has no valid window)
      // Strides 1 and 2: element e is input pixel (ih, iwf + e * sw), so the chunk lies in one window of
      // VEC * sw consecutive pixels.  Pixels left of the row (padding), right of it, and positions past the end
      // of the output row read as zero: elements [lo, hi) are kept.  The window is loaded whole from an address
      // that is always valid; no branch depends on a lane.
      const int sw = g.sw, sft = sw - 1;
      int lo = (sft - iwf) >> sft;            // ceil(-iwf / sw); <= 0 when the window starts inside the row
      int hi = ((g.W - 1 - iwf) >> sft) + 1;  // elements up to the right edge of the row; <= 0 beyond it
      lo = lo < 0 ? 0 : (lo > VEC ? VEC : lo);
      hi = hi < 0 ? 0 : (hi > pcnt ? pcnt : hi);
      if (!row_ok) hi = 0;
      const bool any = hi > lo;
      const bool inside = start >= 0 && start + VEC * sw <= g.numel_x;  // the whole window lies in the tensor
      const T* win = src + ((any && inside) ? start : 0);
      wstart[q] = start;
      winfo[q] = (lo * (VEC + 1) + hi) | ((any && !inside) ? 0x100 : 0);
      wmask[q] = *reinterpret_cast<const u32x4*>(masks + (lo * (VEC + 1) + hi) * 16);
      wsw = sw;
      if (sw == 2) win2[q] = reinterpret_cast<const Unaligned*>(win + VEC)->v;
      return reinterpret_cast<const Unaligned*>(win)->v;
    }
    // Other strides: element e is input pixel (ih, iwf + e * sw), fetched one by one.
    wstart[q] = 0;
    winfo[q] = 0;
    wmask[q] = u32x4{0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
    wsw = 1;
    const int step = g.sw, W = g.W, cnt = row_ok ? pcnt : 0;
    return gather_elements(start, step, [=](int e) { return e < cnt && (unsigned)(iwf + e * step) < (unsigned)W; });
  }

  // Tap-major gather: requests all chunks of the K tile that starts at k0 (k = (kh * KW + kw) * IC + ic; the host
  // guarantees IC % BK == 0, strides of at most 2 and a tensor of at least two chunks).
  __device__ __forceinline__ void request_tile(u32x4 (&regs)[NL], int tid, int k0, const ConvGeom& g) {
    const int kt0 = kofs + k0;
    const int tap = g.d_ic.div(kt0), ic0 = kt0 - tap * g.IC;  // uniform over the workgroup
    const int kh = g.d_kw.div(tap), kw = tap - kh * g.KW;
    const int ih = ih0 + kh, iwf = iw0 + kw;
    const int sw = g.sw, sft = sw - 1;
    int lo = (sft - iwf) >> sft;
    int hi = ((g.W - 1 - iwf) >> sft) + 1;
    lo = lo < 0 ? 0 : (lo > VEC ? VEC : lo);
    hi = hi < 0 ? 0 : (hi > pcnt ? pcnt : hi);
    if ((unsigned)ih >= (unsigned)g.H) hi = 0;
    const bool any = hi > lo;
    tinfo = lo * (VEC + 1) + hi;
    tmask = *reinterpret_cast<const u32x4*>(masks + tinfo * 16);
    wsw = sw;
    tedge = 0u;
    const unsigned base = (unsigned)pofs + (unsigned)(kh * g.W + kw) + (unsigned)ic0 * (unsigned)g.HW;
    const int last = g.numel_x - VEC * sw;
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const int sr = LoadMap::task(tid, q).i;  // channel of the chunk within the tile
      const int start = (int)(base + (unsigned)sr * (unsigned)g.HW);
      const bool inside = start >= 0 && start <= last;
      const T* win = src + ((any && inside) ? start : 0);
      wstart[q] = start;
      if (any && !inside) tedge |= 1u << q;
      if (sw == 2) win2[q] = reinterpret_cast<const Unaligned*>(win + VEC)->v;
      regs[q] = reinterpret_cast<const Unaligned*>(win)->v;
    }
  }

  // The rare forms of the gather (strides above 2, windows at the very ends of the tensor): a rolled loop of
  // predicated single-element loads, small in code and registers because it is off the hot path.
  template <class Pred>
  __device__ __forceinline__ u32x4 gather_elements(int start, int step, Pred ok) const {
    constexpr int HALF = VEC / 2, BITS = 8 * (int)sizeof(T);
    unsigned long long h0 = 0, h1 = 0;
#pragma unroll 1
    for (int e = 0; e < VEC; ++e) {
      if (ok(e)) {
        const T x = src[start + e * step];
        unsigned long long bits;
        if constexpr (IS_F32)
          bits = __builtin_bit_cast(unsigned int, x);
        else
          bits = __builtin_bit_cast(unsigned short, x);
        bits <<= (e % HALF) * BITS;
        if (e < HALF)
          h0 |= bits;
        else
          h1 |= bits;
      }
    }
    return u32x4{(unsigned int)h0, (unsigned int)(h0 >> 32), (unsigned int)h1, (unsigned int)(h1 >> 32)};
  }

  __device__ __forceinline__ u32x4 finish_window(int q, u32x4 v) const {
    if constexpr (MODE == LD_IM2COL_TAP) {
      if (wsw == 2) {
        const u32x4 w = win2[q];
        if constexpr (IS_F32) {
          v = u32x4{v[0], v[2], w[0], w[2]};
        } else {
          v = u32x4{(v[0] & 0xffffu) | (v[1] << 16), (v[2] & 0xffffu) | (v[3] << 16),
                    (w[0] & 0xffffu) | (w[1] << 16), (w[2] & 0xffffu) | (w[3] << 16)};
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] &= tmask[i];
      if (tedge & (1u << q)) {
        const int lo = tinfo / (VEC + 1), hi = tinfo % (VEC + 1);
        v = gather_elements(wstart[q], wsw, [=](int e) { return e >= lo && e < hi; });
      }
      return v;
    }
    const int info = winfo[q];
    if (wsw == 2) {
      const u32x4 w = win2[q];
      if constexpr (IS_F32) {
        v = u32x4{v[0], v[2], w[0], w[2]};
      } else {  // even 16-bit elements of the 16 loaded
        v = u32x4{(v[0] & 0xffffu) | (v[1] << 16), (v[2] & 0xffffu) | (v[3] << 16),
                  (w[0] & 0xffffu) | (w[1] << 16), (w[2] & 0xffffu) | (w[3] << 16)};
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] &= wmask[q][i];
    if (info & 0x100) {
      // first or last pixels of the tensor: the window would have left the allocation (it was read from a
      // valid address instead and is replaced here, element by element)
      const int lo = (info & 0xff) / (VEC + 1), hi = (info & 0xff) % (VEC + 1);
      v = gather_elements(wstart[q], wsw, [=](int e) { return e >= lo && e < hi; });
    }
    return v;
  }

  __device__ __forceinline__ void init(int tid, const ConvGeom& g) {
    if constexpr (GATHER) {
      static_assert(std::is_same<LoadMap, LoadMapRowMajor<SROWS, CPR, NT>>::value, "one chunk column per thread");
      const int sc = LoadMap::task(tid, 0).j * VEC;
      const int p = r0 + sc;                             // GEMM column of element 0
      const int r = g.d_owp.div(p), ow = p - r * g.OWP;  // r = image * OH + oh
      const int img = g.d_oh.div(r), oh = r - img * g.OH;
      ih0 = oh * g.sh - g.ph;
      iw0 = ow * g.sw - g.pw;
      int cnt = g.OW - ow;
      cnt = cnt < rows_left - sc ? cnt : rows_left - sc;
      pcnt = cnt < 0 ? 0 : (cnt > VEC ? VEC : cnt);
      // (a chunk with no real position may lie past the last image, where the offset would leave 32 bits)
      pofs = pcnt > 0 ? (img * g.IC * g.H + ih0) * g.W + iw0 : 0;
    }
    if constexpr (MODE == LD_ELEM) {
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const tmap::Task t = LoadMap::task(tid, q);
        const int sr = t.i, sc = t.j * VEC;
        if constexpr (LAYOUT == L_KC) {
          const int r = sr < rows_left ? sr : rows_left - 1;
          eoff[q] = (long long)r * ld + sc;
          nv[q] = VEC;
        } else {
          const int rem = rows_left - sc;
          int c = sc, n = rem;
          if (rem >= VEC) {
            n = VEC;
          } else if (rem > 0) {
            n = -rem;
          } else {
            n = rows_left >= VEC ? VEC : 0;  // a matrix narrower than one chunk has nowhere to redirect to
            c = rows_left >= VEC ? rows_left - VEC : 0;
          }
          eoff[q] = (long long)sr * ld + c;
          nv[q] = n;
        }
      }
    }
    if constexpr (MODE == LD_VEC) {
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const tmap::Task t = LoadMap::task(tid, q);
        const int sr = t.i, sc = t.j * VEC;
        if constexpr (LAYOUT == L_KC) {
          const int r = sr < rows_left ? sr : rows_left - 1;
          off[q] = r * (int)ld + sc;
        } else {
          const int c = sc + VEC <= rows_left ? sc : rows_left - VEC;
          off[q] = sr * (int)ld + c;
        }
      }
    }
  }

  // Direct global -> LDS loads (16-bit types, plain operands at any element alignment).  Lane l of a wave writes its 16 bytes at
  // LDS[base + 16*l], so the LDS side of the cooperative load is fixed -- thread t's q-th load fills
  // stored position q*NT + t of the tile -- and the swizzle moves to the global side: the thread
  // fetches the logical chunk that belongs at that position.  The instruction is issued through
  // inline assembly and tracked by hand with s_waitcnt vmcnt(n): the schedule that uses it keeps
  // several stages in flight and waits for the oldest only.
  // `in_place` (element-aligned operands): a chunk that sticks out past the last column of an M/N-contiguous
  // operand is read where it lies -- what follows the row's end is the next row, and the columns it fills are never
  // stored -- instead of being moved back to end at the edge, which is only right when whole chunks stick out.
  // The caller keeps such loads away from the operand's last row.
  int doff[NL];
  __device__ __forceinline__ void init_direct(int tid, bool in_place = false) {
    static_assert(std::is_same<LoadMap, LoadMapRowMajor<SROWS, CPR, NT>>::value, "stored positions in row-major order");
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      // the cooperative-load task mapping repeat(NL,1) o spatial(NT/CPR, CPR): task (row, pc) of thread tid is stored
      // position row * CPR + pc = q * NT + tid, which is where the hardware puts this lane's 16 bytes
      const tmap::Task t = LoadMap::task(tid, q);
      const int row = t.i, pc = t.j;
      const int lc = pc ^ ((LAYOUT == L_KC) ? swz_kc<CPR, MI>(row) : swz_mc<CPR, MI>(row));
      if constexpr (LAYOUT == L_KC) {
        const int r = row < rows_left ? row : rows_left - 1;
        doff[q] = r * (int)ld + lc * VEC;
      } else {
        int c = lc * VEC + VEC <= rows_left ? lc * VEC : rows_left - VEC;
        if (in_place) c = lc * VEC < rows_left ? lc * VEC : 0;
        doff[q] = row * (int)ld + c;
      }
    }
  }
  // `tile_lds`: LDS byte address of the tile; `wave`: wave index (both wave-uniform).
  __device__ __forceinline__ void load_direct(unsigned tile_lds, int wave, int k0) const {
    const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const T* g = base + doff[q];
      const unsigned dst = tile_lds + (unsigned)((q * NT + wave * 64) * 16);
      // M0 (the LDS destination of the load) is written here, so it is named as clobbered: the compiler must not
      // keep a value of its own in it across the statement.  It reserves M0 and says so in a warning, silenced here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst) : "memory", "m0");
#pragma clang diagnostic pop
    }
  }

  // A K tile that lies entirely inside the matrix: no predicates at all in vector mode.
  __device__ __forceinline__ void load_full(u32x4 (&regs)[NL], int tid, int k0, const ConvGeom& g) {
    if constexpr (MODE == LD_VEC) {
      const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
#pragma unroll
      for (int q = 0; q < NL; ++q) regs[q] = *reinterpret_cast<const u32x4*>(base + off[q]);
    } else if constexpr (MODE == LD_ELEM) {
      const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const long long o = ((LAYOUT == L_KC) ? (long long)k0 : (long long)k0 * ld) + eoff[q];
        if (nv[q] == VEC || (nv[q] < 0 && o + VEC <= span)) {
          regs[q] = reinterpret_cast<const Unaligned*>(base + eoff[q])->v;
        } else {
          const int cnt = nv[q] < 0 ? -nv[q] : nv[q];
          T tmp[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const bool ok = e < cnt;
            const T v = base[ok ? eoff[q] + e : eoff[q]];
            tmp[e] = ok ? v : (T)0.0f;
          }
          regs[q] = __builtin_bit_cast(u32x4, tmp);
        }
      }
    } else {
      load_edge(regs, tid, k0, g);
    }
  }

  // The last, partial K tile (and every tile of the element-wise modes).
  __device__ __forceinline__ void load_edge(u32x4 (&regs)[NL], int tid, int k0, const ConvGeom& g) {
    if constexpr (MODE == LD_IM2COL_TAP) {
      request_tile(regs, tid, k0, g);
      return;
    }
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const tmap::Task t = LoadMap::task(tid, q);
      const int sr = t.i, sc = t.j * VEC;  // stored row, first stored column of the chunk
      if constexpr (MODE == LD_VEC) {
        const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
        const bool inside = (LAYOUT == L_KC) ? (k0 + sc < K) : (k0 + sr < K);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (inside) v = *reinterpret_cast<const u32x4*>(base + off[q]);
        regs[q] = v;
      } else if constexpr (MODE == LD_IM2COL) {
        regs[q] = request_window(q, sr, k0, g);
      } else {
        regs[q] = gather(sr, sc, k0);
      }
    }
  }

  // ---- registers -> LDS ---------------------------------------------------------------------
  // `relu`: the fused input prologue -- every element passes through f(v) = (v < 0 ? 0 : v) on its way into LDS.
  // A negative value of any of the three types has its sign bit set, i.e. is negative as a signed integer of its
  // width, and a non-negative one is its own integer image: a signed integer max with 0 is that f, two elements per
  // instruction for the 16-bit types.
  __device__ __forceinline__ void store(const u32x4 (&regs)[NL], int tid, unsigned char* tile, bool relu = false) const {
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const tmap::Task t = LoadMap::task(tid, q);
      u32x4 v = regs[q];
      if constexpr (GATHER) v = finish_window(q, v);
      if (relu) {
        if constexpr (IS_F32) {
          typedef int i32x4 __attribute__((ext_vector_type(4)));
          const i32x4 z = {0, 0, 0, 0};
          v = __builtin_bit_cast(u32x4, __builtin_elementwise_max(__builtin_bit_cast(i32x4, v), z));
        } else {
          typedef short i16x8 __attribute__((ext_vector_type(8)));
          const i16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
          v = __builtin_bit_cast(u32x4, __builtin_elementwise_max(__builtin_bit_cast(i16x8, v), z));
        }
      }
      if constexpr (!IS_F32) {
        const int swz = (LAYOUT == L_KC) ? swz_kc<CPR, MI>(t.i) : swz_mc<CPR, MI>(t.i);
        *reinterpret_cast<u32x4*>(tile + (t.i * CPR + (t.j ^ swz)) * 16) = v;
      } else if constexpr (LAYOUT == L_MC) {
        *reinterpret_cast<u32x4*>(tile + (t.i * CPR + t.j) * 16) = v;
      } else {
        // fp32, KC source: row t.i, k = 4*t.j + e  ->  LDS [k][row]
        unsigned int* w = reinterpret_cast<unsigned int*>(tile);
#pragma unroll
        for (int e = 0; e < 4; ++e) w[(t.j * 4 + e) * ROWS + t.i] = v[e];
      }
    }
  }

  // ---- LDS -> MFMA fragment -----------------------------------------------------------------
  // Fragment `f` (rows f*MI .. f*MI+MI-1 of the wave's sub-tile starting at row `w0`), k step `ks`.
  __device__ __forceinline__ Frag fragment(const unsigned char* tile, int lane, int w0, int f, int ks) const {
    if constexpr (IS_F32) {
      const int k = ks * KGROUPS + lane / MI;
      const int r = w0 + f * MI + lane % MI;
      return reinterpret_cast<const float*>(tile)[k * ROWS + r];
    } else if constexpr (LAYOUT == L_KC) {
      const int r = w0 + f * MI + lane % MI;
      const int c = ks * KGROUPS + lane / MI;
      const u32x4 v = *reinterpret_cast<const u32x4*>(tile + (r * CPR + (c ^ swz_kc<CPR, MI>(r))) * 16);
      return __builtin_bit_cast(Frag, v);
    } else {
      // transposing read: within each group of 16 lanes, lane s supplies the address of 4
      // elements (k = kb + s/4, columns cb + 4*(s%4) ..+3) and receives column cb + s, k = kb..kb+3
      const int b = lane / 16, s = lane % 16;
      int kb, cb;
      if constexpr (MI == 32) {
        kb = ks * 16 + 8 * (b / 2);
        cb = w0 + f * 32 + 16 * (b % 2);
      } else {
        kb = ks * 32 + 8 * b;
        cb = w0 + f * 16;
      }
      const int k = kb + s / 4;
      const int col = cb + 4 * (s % 4);
      u32x2 h[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int kk = k + 4 * i;
        const unsigned char* addr = tile + (kk * CPR + ((col / 8) ^ swz_mc<CPR, MI>(kk))) * 16 + (col % 8) * 2;
        const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) i16x4*)(const_cast<unsigned char*>(addr)));
        h[i] = __builtin_bit_cast(u32x2, v);
      }
      const u32x4 v = {h[0][0], h[0][1], h[1][0], h[1][1]};
      return __builtin_bit_cast(Frag, v);
    }
  }
};

}  // namespace hidet
