// S3 + S4: the candidate-evaluation contraction with the loss fused into its
// epilogue (Sec. 3.2.1 objective; Sec. 2.2 smoothing identity), and the same
// contraction with a store epilogue (f_fp of Sec. 3.2.1; PassAct2 output).
//
// The kernels compute  D[o, t] = sum_c What[o, c] * X[t, c]  on fp16/bf16 MFMA
// with float accumulation.  `What` stacks the folded operands
// of all candidates ([n_cand * c_out, c_in]), so the alpha grid is simply an
// extra stretch of the o dimension and every X tile is shared by all
// candidates.  In the loss epilogue each lane owns one token column of its
// accumulator tiles: it subtracts the accumulators from Y_ref, squares, sums
// over its output rows, multiplies by that token's weight and the block
// reduces to ONE float per (candidate, tile).  Candidate outputs never reach
// HBM.
//
// The same kernels serve the second-moment form of the search (gram.hip): the product of the
// transposed, weighted tokens with themselves (store epilogue, only the tiles of one triangle,
// the long contraction split into "candidates" that are summed afterwards), and the quadratic
// form of every candidate's weight error in that matrix (EPI_DOT: accumulator times Y instead of
// the squared residual; SYMK: only the upper part of the symmetric operand is contracted).
//
// Two kernels share the tile epilogues and the block -> tile map:
//   gemm_dma_kernel  the pipelined one (c_in % 64 == 0): 16x16x32 MFMA, operands brought
//                    into LDS by LDS-DMA loads, two 64 KB stages, hand-placed waits;
//   gemm_kernel      the general one: 32x32x16 MFMA, register-staged loads.
// Tiling (wave64): block tile 256 x 256 outputs, k-tile 64; waves own 128 x 64
// sub-tiles.  Both operands are K-contiguous in memory, so a fragment is one
// 16-byte LDS read per lane.  LDS rows are 128 B (64 halves) and the eight
// 16-byte chunks of a row are XOR-swizzled with (row/2)%8 so that the 16 lanes
// served together by a 128-bit LDS access touch 16 different bank groups, for
// the fragment reads and for the tile writes alike.
#include <cstdlib>
#include <utility>

#include "common.h"

namespace tlq {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Mma;
template <> struct Mma<F16> {
  static __device__ __forceinline__ f32x16 run(const uint4& a, const uint4& b, const f32x16& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma<BF16> {
  static __device__ __forceinline__ f32x16 run(const uint4& a, const uint4& b, const f32x16& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16x16x32: half the accumulator registers read and written per flop of the 32x32x16 shape.  The
// matrix cores are power-limited with real operands, and a register-only loop with random operands
// sustains 1840 TFLOP/s with this shape against 1585 with 32x32x16, so the pipelined kernel uses it.
template <typename T> struct Mma16;
template <> struct Mma16<F16> {
  static __device__ __forceinline__ f32x4 run(const uint4& a, const uint4& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma16<BF16> {
  static __device__ __forceinline__ f32x4 run(const uint4& a, const uint4& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

// How a wave's accumulators map to (output row, token).  With either MFMA shape (weights as the
// "A" operand, tokens as "B") a lane owns ONE token column per accumulator tile and groups of four
// consecutive output rows ("quads").  A layout names its quads q < NQ and token blocks tb < NTB:
//   tok(tb, lane)  token of the lane inside the wave tile,
//   row(q, lane)   first of the four output rows of quad q inside the wave tile,
//   get(acc, q, tb, r)  the accumulator of row(q) + r and tok(tb),
//   tok_sum(v)     sum of v over the lanes that hold the same token.
template <int FA, int FB> struct Acc32 {   // acc[FA][FB] of f32x16 (32x32x16)
  static constexpr int NQ = FA * 4, NTB = FB, WO = FA * 32, WT = FB * 32;
  static __device__ __forceinline__ int tok(int tb, int lane) { return tb * 32 + (lane & 31); }
  static __device__ __forceinline__ int row(int q, int lane) { return (q >> 2) * 32 + (q & 3) * 8 + (lane >> 5) * 4; }
  template <typename A> static __device__ __forceinline__ float get(const A& acc, int q, int tb, int r) {
    return acc[q >> 2][tb][(q & 3) * 4 + r];
  }
  static __device__ __forceinline__ float tok_sum(float v) { return v + __shfl_xor(v, 32, 64); }
};
template <int IA, int JB> struct Acc16 {   // acc[IA][JB] of f32x4 (16x16x32)
  static constexpr int NQ = IA, NTB = JB, WO = IA * 16, WT = JB * 16;
  static __device__ __forceinline__ int tok(int tb, int lane) { return tb * 16 + (lane & 15); }
  static __device__ __forceinline__ int row(int q, int lane) { return q * 16 + (lane >> 4) * 4; }
  template <typename A> static __device__ __forceinline__ float get(const A& acc, int q, int tb, int r) {
    return acc[q][tb][r];
  }
  static __device__ __forceinline__ float tok_sum(float v) {
    v += __shfl_xor(v, 16, 64);
    return v + __shfl_xor(v, 32, 64);
  }
};

// EPI_DOT: partial = sum over the tile of acc * Y (Y read like Y_ref, one matrix per candidate, no
// token weights): the quadratic form of the second-moment search.
enum { EPI_LOSS = 0, EPI_LOSS_TOK = 1, EPI_STORE = 2, EPI_DOT = 3 };
constexpr int BK = 64;        // halves per k-tile
constexpr int ROWB = BK * 2;  // bytes per LDS row
// An L2 patch (one per XCD at a time) is po x pt tiles = 32 workgroups: 4 x 8 by default (4 operand
// panels that stay while the walk moves along the tokens + 8 token panels), or 8 x 4 for launches
// whose walk keeps the output-side panels and changes the token-side ones from patch to patch.
constexpr int PATCH_SLOTS = 32, kXcd = 8;

struct GemmDev {
  const uint16_t* X; int64_t n_tok, c_in, ldx, x_cand_stride;
  const float* tok_scale;  // [n_cand, n_tok] per-token factor on the accumulators, or NULL
  const uint16_t* Wh; int64_t c_out, ldw, w_cand_stride; int n_cand;
  const void* Yref; int64_t ldy; int ydt; const float* token_w;
  int64_t y_cand_stride;   // elements between per-candidate Y matrices (EPI_DOT; 0 = shared)
  int tri;                 // 1: only tiles with tile row <= tile column are computed (symmetric product)
  int cand_outer;          // 1: the candidate is the outermost level of the block order
  int64_t o_cand_stride;   // EPI_STORE: elements between per-candidate outputs
  float* partial; float* tok_partial;
  void* Yout; int64_t ldo; int odt;
  int tiles_o, tiles_t, npo, npt;  // tiles per candidate and patches per candidate
  int64_t n_patches;
  int cpt;          // token patches per chunk (see make_dev)
  int rag, rag_pt;  // tile rows of the last, incomplete patch row (0 = none) and its patch width in tiles
  int po, pt;       // patch shape in tiles (po * pt == PATCH_SLOTS)
};

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ float load_y(const void* Y, int ydt, int64_t idx) {
  if (ydt == TLQ_F32) return ((const float*)Y)[idx];
  const uint16_t b = ((const uint16_t*)Y)[idx];
  return ydt == TLQ_F16 ? F16::to_float(b) : BF16::to_float(b);
}
__device__ __forceinline__ void load_y4(const void* Y, int ydt, int64_t idx, float y[4]) {
  if (ydt == TLQ_F32) {
    const float4 v = *reinterpret_cast<const float4*>((const float*)Y + idx);
    y[0] = v.x; y[1] = v.y; y[2] = v.z; y[3] = v.w;
  } else {
    const uint2 v = *reinterpret_cast<const uint2*>((const uint16_t*)Y + idx);
    if (ydt == TLQ_F16) {
      y[0] = F16::to_float((uint16_t)v.x); y[1] = F16::to_float((uint16_t)(v.x >> 16));
      y[2] = F16::to_float((uint16_t)v.y); y[3] = F16::to_float((uint16_t)(v.y >> 16));
    } else {
      y[0] = BF16::to_float((uint16_t)v.x); y[1] = BF16::to_float((uint16_t)(v.x >> 16));
      y[2] = BF16::to_float((uint16_t)v.y); y[3] = BF16::to_float((uint16_t)(v.y >> 16));
    }
  }
}
__device__ __forceinline__ void store_y4(void* Y, int odt, int64_t idx, const float y[4]) {
  if (odt == TLQ_F32) {
    *reinterpret_cast<float4*>((float*)Y + idx) = make_float4(y[0], y[1], y[2], y[3]);
  } else if (odt == TLQ_F16) {
    *reinterpret_cast<uint2*>((uint16_t*)Y + idx) =
        make_uint2((uint32_t)F16::from_float(y[0]) | ((uint32_t)F16::from_float(y[1]) << 16),
                   (uint32_t)F16::from_float(y[2]) | ((uint32_t)F16::from_float(y[3]) << 16));
  } else {
    *reinterpret_cast<uint2*>((uint16_t*)Y + idx) =
        make_uint2((uint32_t)BF16::from_float(y[0]) | ((uint32_t)BF16::from_float(y[1]) << 16),
                   (uint32_t)BF16::from_float(y[2]) | ((uint32_t)BF16::from_float(y[3]) << 16));
  }
}
__device__ __forceinline__ void store_y1(void* Y, int odt, int64_t idx, float y) {
  if (odt == TLQ_F32) ((float*)Y)[idx] = y;
  else ((uint16_t*)Y)[idx] = odt == TLQ_F16 ? F16::from_float(y) : BF16::from_float(y);
}



// Per-lane part of the loss of one wave tile whose first output row is `ow` and first
// token is `tw`: sq[tb] = sum over this lane's rows of (Y_ref - acc)^2 for its token of
// token block tb; part = sum_tb token_w * sq[tb].  YDT >= 0 fixes the Y_ref type at
// compile time; FULL promises that the whole wave tile lies inside the matrix.
// DOT replaces the squared residual by the product acc * y and drops the token weight.
template <int YDT, bool FULL, bool DOT, typename L, typename Acc>
__device__ __forceinline__ void loss_rows(const GemmDev& a, const void* Yref, const Acc& acc, const float* tsc,
                                          int64_t ow, int64_t tw, float (&sq)[L::NTB], float& part) {
  const int lane = threadIdx.x & 63;
  const int ydt = YDT >= 0 ? YDT : a.ydt;
#pragma unroll
  for (int tb = 0; tb < L::NTB; ++tb) {
    const int64_t t = tw + L::tok(tb, lane);
    float sumsq = 0.0f;
    if (FULL || t < a.n_tok) {
      // residual = y - sg * acc as one fused multiply-add; sg = 1 gives y - acc exactly
      const float nsg = tsc ? -tsc[t] : -1.0f;
#pragma unroll
      for (int q = 0; q < L::NQ; ++q) {
        const int64_t o = ow + L::row(q, lane);
        if (FULL || o + 3 < a.c_out) {
          float y[4];
          load_y4(Yref, ydt, t * a.ldy + o, y);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (DOT) { sumsq += L::get(acc, q, tb, r) * y[r]; continue; }
            const float d = __builtin_fmaf(nsg, L::get(acc, q, tb, r), y[r]);
            sumsq += d * d;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (o + r < a.c_out) {
              const float y = load_y(Yref, ydt, t * a.ldy + o + r);
              if (DOT) { sumsq += L::get(acc, q, tb, r) * y; continue; }
              const float d = __builtin_fmaf(nsg, L::get(acc, q, tb, r), y);
              sumsq += d * d;
            }
        }
      }
      part += DOT ? sumsq : a.token_w[t] * sumsq;
    }
    sq[tb] = sumsq;
  }
}

// Same sums as loss_rows for an interior wave tile with 16-bit Y_ref, but Y_ref goes through
// LDS: the wave copies its 64-token x 128-row piece with whole-line loads (each 128-byte line
// is fetched once, 8 lines per instruction) into `ylds` (WT x WO 16-bit, this wave's own),
// then every lane picks its values from there.  Reading Y_ref straight from the accumulator
// layout touches 16 or 32 lines per instruction and each line 8 times.  16-byte chunks of a token
// row are stored at chunk ^ (token % 16), which makes the 8-byte reads conflict-free.
template <typename YT, bool DOT, typename L, typename Acc>
__device__ __forceinline__ void loss_rows_lds(const GemmDev& a, const void* Yref, const Acc& acc, const float* tsc,
                                              int64_t ow, int64_t tw, float (&sq)[L::NTB], float& part,
                                              unsigned char* ylds) {
  constexpr int WO = L::WO, WT = L::WT;
  constexpr int CPR = WO / 8;              // 16-byte chunks per token row
  constexpr int RPI = 64 / CPR;            // token rows per wave-wide copy
  static_assert(CPR == 16 && WT % RPI == 0, "copy shape");
  const int lane = threadIdx.x & 63;
  const uint16_t* Y = (const uint16_t*)Yref;
  {
    const int cr = lane / CPR, cc = lane % CPR;
    uint4 v[WT / RPI];
#pragma unroll
    for (int j = 0; j < WT / RPI; ++j) {
      const int row = j * RPI + cr;
      v[j] = *reinterpret_cast<const uint4*>(Y + (tw + row) * a.ldy + ow + cc * 8);
    }
#pragma unroll
    for (int j = 0; j < WT / RPI; ++j) {
      const int row = j * RPI + cr;
      *reinterpret_cast<uint4*>(ylds + row * (WO * 2) + ((cc ^ (row & 15)) << 4)) = v[j];
    }
  }
  // the values are picked up by OTHER lanes of this wave: order the LDS writes before the reads
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int tb = 0; tb < L::NTB; ++tb) {
    const int tok = L::tok(tb, lane);
    const int64_t t = tw + tok;
    const float nsg = tsc ? -tsc[t] : -1.0f;
    float sumsq = 0.0f;
#pragma unroll
    for (int q = 0; q < L::NQ; ++q) {
      const int o = L::row(q, lane);        // multiple of 4: chunk o / 8, half (o / 4) % 2
      const uint2 u = *reinterpret_cast<const uint2*>(ylds + tok * (WO * 2) + (((o >> 3) ^ (tok & 15)) << 4) +
                                                      ((o >> 2) & 1) * 8);
      const float y[4] = {YT::to_float((uint16_t)(u.x & 0xffffu)), YT::to_float((uint16_t)(u.x >> 16)),
                          YT::to_float((uint16_t)(u.y & 0xffffu)), YT::to_float((uint16_t)(u.y >> 16))};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (DOT) { sumsq += L::get(acc, q, tb, r) * y[r]; continue; }
        const float d = __builtin_fmaf(nsg, L::get(acc, q, tb, r), y[r]);
        sumsq += d * d;
      }
    }
    part += DOT ? sumsq : a.token_w[t] * sumsq;
    sq[tb] = sumsq;
  }
}

// Store epilogue of an interior wave tile with a 16-bit output, through LDS: every lane drops
// its rounded values into `ylds` (WT x WO 16-bit, this wave's own, same chunk-XOR-token layout
// as loss_rows_lds), then the wave writes whole 128-byte lines, 8 lines per instruction.
// Storing straight from the accumulator layout writes 8-byte pieces of 16 or 32 lines per instruction.
template <typename YT, typename L, typename Acc>
__device__ __forceinline__ void store_rows_lds(const GemmDev& a, void* Yout, const Acc& acc, const float* tsc,
                                               int64_t ow, int64_t tw, unsigned char* ylds) {
  constexpr int WO = L::WO, WT = L::WT;
  constexpr int CPR = WO / 8, RPI = 64 / CPR;
  static_assert(CPR == 16 && WT % RPI == 0, "copy shape");
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int tb = 0; tb < L::NTB; ++tb) {
    const int tok = L::tok(tb, lane);
    const float sg = tsc ? tsc[tw + tok] : 1.0f;
#pragma unroll
    for (int q = 0; q < L::NQ; ++q) {
      const int o = L::row(q, lane);
      uint2 u;
      u.x = (uint32_t)YT::from_float(sg * L::get(acc, q, tb, 0)) | ((uint32_t)YT::from_float(sg * L::get(acc, q, tb, 1)) << 16);
      u.y = (uint32_t)YT::from_float(sg * L::get(acc, q, tb, 2)) | ((uint32_t)YT::from_float(sg * L::get(acc, q, tb, 3)) << 16);
      *reinterpret_cast<uint2*>(ylds + tok * (WO * 2) + (((o >> 3) ^ (tok & 15)) << 4) + ((o >> 2) & 1) * 8) = u;
    }
  }
  uint16_t* Y = (uint16_t*)Yout;
  const int cr = lane / CPR, cc = lane % CPR;
  // whole lines are read back by OTHER lanes of this wave: order the LDS writes before the reads
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int j = 0; j < WT / RPI; ++j) {
    const int row = j * RPI + cr;
    const uint4 v = *reinterpret_cast<const uint4*>(ylds + row * (WO * 2) + ((cc ^ (row & 15)) << 4));
    *reinterpret_cast<uint4*>(Y + (tw + row) * a.ldo + ow + cc * 8) = v;
  }
}

// ---------------------------------------------------------------------------
// Tile epilogue shared by both kernels; L is the accumulator layout (Acc32 / Acc16).  The block's
// waves form an NWO x NWT grid; wave (wo, wt) owns output rows [wo*WO, +WO) and tokens
// [wt*WT, +WT) of the tile at (o0, t0).  `red` holds one float per wave, `rows` NWO x BT floats
// (per-token row sums; only used by EPI_LOSS_TOK).  Every wave of the block must call this.
template <int EPI, typename L, int NWO, int NWT, int BT, bool YLDS, typename Acc>
__device__ __forceinline__ void tile_epilogue(const GemmDev& a, const Acc& acc, int cand, int to,
                                              int tt, int64_t o0, int64_t t0, int wo, int wt,
                                              float* red, float* rows) {
  constexpr int WO = L::WO, WT = L::WT, NW = NWO * NWT, NT = NW * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* tsc = a.tok_scale ? a.tok_scale + (int64_t)cand * a.n_tok : nullptr;
  if (EPI == EPI_STORE) {
    void* Yo = (unsigned char*)a.Yout + (int64_t)cand * a.o_cand_stride * (a.odt == TLQ_F32 ? 4 : 2);
    if constexpr (YLDS) {
      if (a.odt != TLQ_F32 && (o0 + NWO * WO <= a.c_out) && (t0 + BT <= a.n_tok) && (a.ldo % 8) == 0 &&
          ((uintptr_t)Yo % 16) == 0) {
        unsigned char* ylds = reinterpret_cast<unsigned char*>(rows) + wave * (WO * WT * 2);
        if (a.odt == TLQ_F16) store_rows_lds<F16, L>(a, Yo, acc, tsc, o0 + wo * WO, t0 + wt * WT, ylds);
        else store_rows_lds<BF16, L>(a, Yo, acc, tsc, o0 + wo * WO, t0 + wt * WT, ylds);
        return;
      }
    }
#pragma unroll
    for (int tb = 0; tb < L::NTB; ++tb) {
      const int64_t t = t0 + wt * WT + L::tok(tb, lane);
      if (t >= a.n_tok) continue;
      const float sg = tsc ? tsc[t] : 1.0f;
#pragma unroll
      for (int q = 0; q < L::NQ; ++q) {
        const int64_t o = o0 + wo * WO + L::row(q, lane);
        float y[4] = {sg * L::get(acc, q, tb, 0), sg * L::get(acc, q, tb, 1), sg * L::get(acc, q, tb, 2),
                      sg * L::get(acc, q, tb, 3)};
        if (o + 3 < a.c_out) store_y4(Yo, a.odt, t * a.ldo + o, y);
        else
          for (int r = 0; r < 4; ++r)
            if (o + r < a.c_out) store_y1(Yo, a.odt, t * a.ldo + o + r, y[r]);
      }
    }
    return;
  }
  // Interior tiles (the common case) take a branch-free body specialised on the Y_ref
  // type; edge tiles and odd strides take the guarded one.
  float part = 0.0f;
  float sq[L::NTB];
  const bool interior = (o0 + NWO * WO <= a.c_out) && (t0 + BT <= a.n_tok);
  const int64_t ow = o0 + wo * WO, tw = t0 + wt * WT;
  constexpr bool DOT = EPI == EPI_DOT;
  const void* Yc = a.Yref;
  if (DOT) Yc = (const unsigned char*)a.Yref + (int64_t)cand * a.y_cand_stride * (a.ydt == TLQ_F32 ? 4 : 2);
  bool done = false;
  if constexpr (YLDS && (EPI == EPI_LOSS || DOT)) {
    if (interior && a.ydt != TLQ_F32 && (a.ldy % 8) == 0 && ((uintptr_t)Yc % 16) == 0) {
      unsigned char* ylds = reinterpret_cast<unsigned char*>(rows) + wave * (WO * WT * 2);
      if (a.ydt == TLQ_F16) loss_rows_lds<F16, DOT, L>(a, Yc, acc, tsc, ow, tw, sq, part, ylds);
      else loss_rows_lds<BF16, DOT, L>(a, Yc, acc, tsc, ow, tw, sq, part, ylds);
      done = true;
    }
  }
  if (done) {}
  else if (interior && a.ydt == TLQ_F16) loss_rows<TLQ_F16, true, DOT, L>(a, Yc, acc, tsc, ow, tw, sq, part);
  else if (interior && a.ydt == TLQ_F32) loss_rows<TLQ_F32, true, DOT, L>(a, Yc, acc, tsc, ow, tw, sq, part);
  else if (interior) loss_rows<TLQ_BF16, true, DOT, L>(a, Yc, acc, tsc, ow, tw, sq, part);
  else loss_rows<-1, false, DOT, L>(a, Yc, acc, tsc, ow, tw, sq, part);
  if (EPI == EPI_LOSS_TOK) {
#pragma unroll
    for (int tb = 0; tb < L::NTB; ++tb) {
      const float both = L::tok_sum(sq[tb]);
      if (L::row(0, lane) == 0) rows[wo * BT + wt * WT + L::tok(tb, lane)] = both;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off, 64);
  if (lane == 0) red[wave] = part;
  __syncthreads();
  if (tid == 0) {
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[w];
    a.partial[((int64_t)cand * a.tiles_o + to) * a.tiles_t + tt] = s;
  }
  if (EPI == EPI_LOSS_TOK) {
    for (int i = tid; i < BT; i += NT) {
      const int64_t t = t0 + i;
      if (t < a.n_tok) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NWO; ++w) s += rows[w * BT + i];
        a.tok_partial[(int64_t)to * a.n_tok + t] = s;
      }
    }
  }
}

// Block id -> (candidate, tile row, tile column).  Blocks are dealt to the 8 XCDs round-robin by
// block id, so block id = (round, xcd, slot) and every XCD works on one patch of po x pt tiles at a
// time (32 CUs = 32 tiles sharing, by default, 4 weight panels and 8 token panels in its L2).
// Patch order: chunks of cpt token patches; inside a chunk, for every output patch row, every
// candidate visits the chunk's token patches.  The chunk's tokens and the row's slice of Y_ref are
// thus shared by all candidates while they are hot in the last-level cache, and each candidate's
// weights are streamed once per chunk.  When tiles_o is not a multiple of po the last patch row
// has `rag` tile rows and uses patches of rag x rag_pt tiles, so that (nearly) every slot of a patch
// is a live tile.  Returns false for a slot that has no tile.
__host__ __device__ __forceinline__ bool decode_tile(const GemmDev& a, int64_t bid, int& cand, int& to, int& tt) {
  const int PATCH_O = a.po, PATCH_T = a.pt;
  const int64_t round = bid / (kXcd * PATCH_SLOTS);
  const int within = (int)(bid % (kXcd * PATCH_SLOTS));
  int64_t patch = round * kXcd + (within & (kXcd - 1));
  const int slot = within / kXcd;
  if (patch >= a.n_patches) return false;
  // candidate-outermost order: the same walk with one candidate, repeated per candidate
  int n_cand = a.n_cand, cand0 = 0;
  if (a.cand_outer) {
    const int64_t per = a.n_patches / a.n_cand;
    cand0 = (int)(patch / per);
    patch %= per;
    n_cand = 1;
  }
  const int n_full = a.rag ? a.npo - 1 : a.npo;
  const int ragp_full = a.rag ? (a.cpt * PATCH_T + a.rag_pt - 1) / a.rag_pt : 0;
  const int64_t chunk_sz = (int64_t)n_cand * (n_full * a.cpt + ragp_full);
  const int chunk = (int)(patch / chunk_sz);
  const int crem = (int)(patch % chunk_sz);
  const int cw = (a.npt - chunk * a.cpt) < a.cpt ? (a.npt - chunk * a.cpt) : a.cpt;
  const int nfull_p = n_full * n_cand * cw;
  if (crem < nfull_p) {
    const int r2 = crem % (n_cand * cw);
    cand = cand0 + r2 / cw;
    to = (crem / (n_cand * cw)) * PATCH_O + (slot % PATCH_O);
    tt = (chunk * a.cpt + r2 % cw) * PATCH_T + (slot / PATCH_O);
  } else {
    const int ragp = (cw * PATCH_T + a.rag_pt - 1) / a.rag_pt;
    const int r2 = crem - nfull_p, col = slot / a.rag;
    cand = cand0 + r2 / ragp;
    if (col >= a.rag_pt) return false;
    to = n_full * PATCH_O + (slot % a.rag);
    tt = chunk * a.cpt * PATCH_T + (r2 % ragp) * a.rag_pt + col;
    if (tt >= (chunk * a.cpt + cw) * PATCH_T) return false;
  }
  return to < a.tiles_o && tt < a.tiles_t;
}

// General kernel: two LDS stages; the global loads of k-tile i+1 are issued before the MFMAs of
// k-tile i and written to the other stage afterwards; one barrier per k-tile.
template <typename T, int BO, int BT, int WO, int WT, int EPI>
__global__ __launch_bounds__((BO / WO) * (BT / WT) * 64) void gemm_kernel(GemmDev a) {
  constexpr int NWO = BO / WO, NWT = BT / WT, NW = NWO * NWT, NT = NW * 64;
  constexpr int FA = WO / 32, FB = WT / 32;
  constexpr int CH_A = BO * 8 / NT, CH_B = BT * 8 / NT;  // 16-byte chunks per thread per k-tile
  static_assert(BO * 8 % NT == 0 && BT * 8 % NT == 0, "tile/thread mismatch");
  constexpr int STAGE = (BO + BT) * ROWB;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE];
  __shared__ float red[NW];

  int cand, to, tt;
  if (!decode_tile(a, blockIdx.x, cand, to, tt)) return;
  if (a.tri && to > tt) return;   // the mirrored tile carries the same values
  const int64_t o0 = (int64_t)to * BO, t0 = (int64_t)tt * BT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wo = wave % NWO, wt = wave / NWO;
  const uint16_t* Wc = a.Wh + (int64_t)cand * a.w_cand_stride;

  // ---- global -> register staging
  const uint16_t* pa[CH_A]; bool oka[CH_A]; int la[CH_A];
  const uint16_t* pb[CH_B]; bool okb[CH_B]; int lb[CH_B];
  const int lchunk = tid & 7;
#pragma unroll
  for (int i = 0; i < CH_A; ++i) {
    const int r = (i * NT + tid) >> 3;
    oka[i] = (o0 + r) < a.c_out;
    pa[i] = Wc + (oka[i] ? (o0 + r) : 0) * a.ldw + lchunk * 8;
    la[i] = r * ROWB + (swz(r, lchunk) << 4);
  }
#pragma unroll
  for (int i = 0; i < CH_B; ++i) {
    const int r = (i * NT + tid) >> 3;
    okb[i] = (t0 + r) < a.n_tok;
    pb[i] = a.X + (int64_t)cand * a.x_cand_stride + (okb[i] ? (t0 + r) : 0) * a.ldx + lchunk * 8;
    lb[i] = BO * ROWB + r * ROWB + (swz(r, lchunk) << 4);
  }
  uint4 ga[CH_A], gb[CH_B];
  auto gload = [&](int64_t k0) {
    const bool kok = (k0 + lchunk * 8) < a.c_in;
#pragma unroll
    for (int i = 0; i < CH_A; ++i) {
      ga[i] = make_uint4(0, 0, 0, 0);
      if (oka[i] && kok) ga[i] = *reinterpret_cast<const uint4*>(pa[i] + k0);
    }
#pragma unroll
    for (int i = 0; i < CH_B; ++i) {
      gb[i] = make_uint4(0, 0, 0, 0);
      if (okb[i] && kok) gb[i] = *reinterpret_cast<const uint4*>(pb[i] + k0);
    }
  };
  auto lstore = [&](int stage) {
    unsigned char* base = lds + stage * STAGE;
#pragma unroll
    for (int i = 0; i < CH_A; ++i) *reinterpret_cast<uint4*>(base + la[i]) = ga[i];
#pragma unroll
    for (int i = 0; i < CH_B; ++i) *reinterpret_cast<uint4*>(base + lb[i]) = gb[i];
  };

  // ---- fragment read offsets: lane -> row (lane%32), k-chunk (lane/32) + 2*kk
  const int frow = lane & 31, fhi = lane >> 5;
  int offk[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) offk[kk] = frow * ROWB + (swz(frow, kk * 2 + fhi) << 4);
  const int a_base = (wo * WO) * ROWB;
  const int b_base = BO * ROWB + (wt * WT) * ROWB;

  f32x16 acc[FA][FB];
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int64_t nk = (a.c_in + BK - 1) / BK;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int cur = (int)(kt & 1);
    if (kt + 1 < nk) gload((kt + 1) * BK);
    const unsigned char* sb = lds + cur * STAGE;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 fa[FA], fb[FB];
#pragma unroll
      for (int i = 0; i < FA; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(sb + a_base + i * 32 * ROWB + offk[kk]);
#pragma unroll
      for (int j = 0; j < FB; ++j)
        fb[j] = *reinterpret_cast<const uint4*>(sb + b_base + j * 32 * ROWB + offk[kk]);
#pragma unroll
      for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j) acc[i][j] = Mma<T>::run(fa[i], fb[j], acc[i][j]);
    }
    if (kt + 1 < nk) lstore(cur ^ 1);
    __syncthreads();
  }

  // the tile memory is free now: row sums of the per-token variant reuse it
  tile_epilogue<EPI, Acc32<FA, FB>, NWO, NWT, BT, false>(a, acc, cand, to, tt, o0, t0, wo, wt, red,
                                                         reinterpret_cast<float*>(lds));
}

// ---------------------------------------------------------------------------
// Pipelined variant for c_in % BK == 0 (every group-128 workload).
//
// Global -> LDS goes through the buffer-load-to-LDS path (no VGPR staging, no
// LDS store instructions): each wave-wide load drops 64 x 16 B contiguously at
// an LDS base held in M0, so the XOR swizzle is applied on the *global* side
// (lane l fetches the chunk that belongs in LDS slot l).  Rows past the edge
// of the matrix fall outside the buffer descriptor's range and arrive as
// zeros.  NSTAGE k-tiles form a ring; the refill of a slot is issued as soon
// as the block-wide barrier shows that every wave has finished reading it, so
// NSTAGE-1 k-tiles of loads are always in flight.
//
// The compiler cannot see that fragment reads and LDS-DMA writes touch
// different ring slots and would drain the load counter before every LDS read,
// so the fragment reads are issued from inline assembly and the waits on the
// two counters are placed by hand:
//   - "lgkmcnt(0)" ties the fragment registers, so no MFMA can be scheduled
//     before its operands have arrived;
//   - "vmcnt(n)" before the barrier waits for this wave's share of the next
//     k-tile only.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int IMM>
__device__ __forceinline__ void lds_read128(u32x4& v, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM));
}
// Wait for every outstanding LDS read; the fragments are tied through the
// statement so that nothing consuming them can be scheduled above it.
__device__ __forceinline__ void lds_wait4(u32x4& f0, u32x4& f1, u32x4& f2, u32x4& f3) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f0), "+v"(f1), "+v"(f2), "+v"(f3) : : "memory");
}
__device__ __forceinline__ void lds_wait8(u32x4& f0, u32x4& f1, u32x4& f2, u32x4& f3, u32x4& f4,
                                          u32x4& f5, u32x4& f6, u32x4& f7) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f0), "+v"(f1), "+v"(f2), "+v"(f3), "+v"(f4), "+v"(f5), "+v"(f6), "+v"(f7)
               :
               : "memory");
}
template <int I, int N, typename Fn>
__device__ __forceinline__ void static_for(Fn&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Block tile 256 (o) x 256 (t), k-tile 64, 8 waves in a 2 x 4 grid; a wave owns 128 x 64 outputs
// = 8 x 4 accumulator tiles of the 16x16x32 MFMA (128 registers).  A k-tile is two k32 steps; a
// step is split into two PHASES of 16 MFMAs (output rows 0-63, then 64-127 of the wave tile), so
// only four weight fragments and four token fragments are live per phase and both sets can be
// double-buffered in 64 registers:
//   phase 0: rows  0-63  x step 0   reads meanwhile: weight fragments of rows 64-127, step 0
//   phase 1: rows 64-127 x step 0   reads meanwhile: weight fragments of rows 0-63 and the token
//                                   fragments of step 1
//   phase 2: rows  0-63  x step 1   reads meanwhile: weight fragments of rows 64-127, step 1
//   -- every fragment of the k-tile is in registers: wait for this wave's loads of the next
//      k-tile, block barrier --
//   phase 3: rows 64-127 x step 1   reads meanwhile: first fragments of the NEXT k-tile; the 8
//                                   LDS-DMA loads that refill the slot just freed
// The side operations are slotted two at a time behind the first MFMAs of a phase (measured best:
// one per MFMA over the whole phase -3 %, four at a time -2 %), so that neither the LDS queue nor
// the texture-address queue sees a burst that would hold back the in-order MFMA issue.
// SYMK: Wh is a symmetric square matrix (c_out == c_in) and the epilogue forms a quadratic form in
// it (EPI_DOT with Y == X): the tile with first output row o0 contracts only k >= o0, with the part
// beyond its diagonal block counted twice: 2 * sum_{k > block} + sum_{k in block} stands for the
// full contraction at about half the flops.  The k-tiles are walked from the END of the rows
// down to o0, so that the tiles of a patch - which start at different o0 - work on the same
// k-tile at the same time and share its token panel in L2; the diagonal block comes last.
template <typename T, int NSTAGE, int EPI, bool SYMK = false>
__global__ __launch_bounds__(512) void gemm_dma_kernel(GemmDev a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the body uses gfx950 builtins the host pass cannot parse
  constexpr int BK_ = 64, BO = 256, BT = 256, NWO = 2, NWT = 4, NW = NWO * NWT, WO = BO / NWO, WT = BT / NWT;
  constexpr int IA = WO / 16, JB = WT / 16;   // accumulator tiles per wave: 8 x 4
  static_assert(IA == 8 && JB == 4, "phase structure below is written for 128 x 64 wave tiles");
  constexpr int RB = BK_ * 2;             // bytes per LDS row
  constexpr int CPR = BK_ / 8;            // 16-byte chunks per row
  constexpr int STAGE = (BO + BT) * RB;
  constexpr int RPD = 64 / CPR;           // rows covered by one wave-wide load
  constexpr int DPO = BO / RPD / NW;      // loads per wave per operand per k-tile
  constexpr int LPS = 2 * DPO;            // loads per wave per k-tile
  static_assert(NSTAGE == 2 && LPS == 8, "pipeline shape");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[NSTAGE * STAGE];
  __shared__ float red[NW];

  int cand, to, tt;
  if (!decode_tile(a, blockIdx.x, cand, to, tt)) return;
  if (a.tri && to > tt) return;   // the mirrored tile carries the same values
  const int64_t o0 = (int64_t)to * BO, t0 = (int64_t)tt * BT;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = wave % NWO, wt = wave / NWO;

  // buffer descriptors over the valid rows of this block's two operand panels
  const int64_t vro = (a.c_out - o0) < BO ? (a.c_out - o0) : BO;
  const int64_t vrt = (a.n_tok - t0) < BT ? (a.n_tok - t0) : BT;
  const int64_t kskip = SYMK ? o0 : 0;    // first contraction index (a multiple of the tile height)
  const int64_t klen = a.c_in - kskip;
  const uint16_t* pA = a.Wh + (int64_t)cand * a.w_cand_stride + o0 * a.ldw + kskip;
  const uint16_t* pB = a.X + (int64_t)cand * a.x_cand_stride + t0 * a.ldx + kskip;
  const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(
      (void*)pA, 0, (int)(((vro - 1) * a.ldw + klen) * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(
      (void*)pB, 0, (int)(((vrt - 1) * a.ldx + klen) * 2), 0x00020000);

  // per-lane global byte offsets of the chunks this lane fetches: LDS slot `p` of row r holds
  // chunk p ^ ((r / 2) % 8)
  int voa[DPO], vob[DPO];
#pragma unroll
  for (int j = 0; j < DPO; ++j) {
    const int r = (j * NW + wave) * RPD + lane / CPR;
    const int p = lane % CPR;
    const int c = p ^ ((r >> 1) & 7);
    voa[j] = r * (int)a.ldw * 2 + c * 16;
    vob[j] = r * (int)a.ldx * 2 + c * 16;
  }
  // The scalar offset is not part of the descriptor's range check, so a k-tile
  // past the end of the rows must not be fetched at all: its loads are still
  // issued (the counter bookkeeping stays uniform) but with a per-lane offset
  // that is out of range for any descriptor, which touches no memory and
  // delivers zeros.
  const int64_t nk = klen / BK_;
  constexpr int kOutOfRange = (int)0x80000000u;
  auto dma1 = [&](auto dc, unsigned char* sbase, bool live, int so) {
    constexpr int d = decltype(dc)::value, j = d / 2;
    if constexpr ((d & 1) == 0)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, (lds_ptr_t)(sbase + (j * NW + wave) * 1024), 16,
                                               live ? voa[j] : kOutOfRange, so, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rB, (lds_ptr_t)(sbase + BO * RB + (j * NW + wave) * 1024), 16,
                                               live ? vob[j] : kOutOfRange, so, 0, 0);
  };
  // byte offset of k-tile number kt of the walk inside a row
  auto k_offset = [&](int64_t kt) { return (int)((SYMK ? nk - 1 - kt : kt) * BK_ * 2); };
  auto issue = [&](int64_t kt) {
    const bool live = kt < nk;
    const int so = live ? k_offset(kt) : 0;
    unsigned char* sb = lds + (int)(kt % NSTAGE) * STAGE;
    static_for<0, LPS>([&](auto dc) { dma1(dc, sb, live, so); });
  };

  // fragment read addresses (bytes from the start of a stage): lane -> row lane % 16 of a 16-row
  // block and 16-byte chunk lane / 16 of the k32 step (the MFMA takes k = 8 * (lane / 16) + [0, 8)
  // from both operands, so any chunk order is right as long as both use the same one)
  const int frow = lane & 15, fq = lane >> 4;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  uint32_t offA[2], offB[2];
#pragma unroll
  for (int st = 0; st < 2; ++st) {
    const int c = st * 4 + fq;
    const int p = c ^ ((frow >> 1) & 7);
    const uint32_t o = (uint32_t)(frow * RB + p * 16);
    offA[st] = lds0 + o + (wo * WO) * RB;
    offB[st] = lds0 + o + BO * RB + (wt * WT) * RB;
  }
  u32x4 Fa[2][4], Fb[2][4];   // weight fragments (double-buffered per phase), token fragments (per k32 step)
  f32x4 acc[IA][JB];
#pragma unroll
  for (int i = 0; i < IA; ++i)
#pragma unroll
    for (int j = 0; j < JB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;

  // One phase: the 16 MFMAs of weight buffer AB x token buffer BB into output rows HALF, with the
  // side operations behind the first eight: the weight fragments of half RH into buffer AB ^ 1
  // (from `ra`), - if RDB - the token fragments into buffer BB ^ 1 (from `rb`), and ND LDS-DMA
  // loads of k-tile `dkt`.
  auto phase = [&](auto abc, auto bbc, auto halfc, auto rhc, auto rdbc, auto ndc, uint32_t ra, uint32_t rb,
                   int64_t dkt) {
    constexpr int AB = decltype(abc)::value, BB = decltype(bbc)::value, HALF = decltype(halfc)::value;
    constexpr int RH = decltype(rhc)::value, ND = decltype(ndc)::value;
    constexpr bool RDB = decltype(rdbc)::value != 0;
    constexpr int NR = 4 + (RDB ? 4 : 0);
    static_assert(NR + ND <= 16, "two side operations behind each of the first eight MFMAs");
    const bool live = dkt < nk;
    const int so = live ? k_offset(dkt) : 0;
    unsigned char* sbase = lds + (int)(dkt % NSTAGE) * STAGE;
    // side operation number n of the phase: in the refill phase the LDS-DMA loads come first (the
    // longest latency), then the fragment reads
    auto side = [&](auto nc) {
      constexpr int n0 = decltype(nc)::value;
      constexpr int n = ND > 0 ? (n0 < ND ? NR + n0 : n0 - ND) : n0;
      if constexpr (n < 4) lds_read128<(RH * 4 + n) * 16 * RB>(Fa[AB ^ 1][n], ra);
      else if constexpr (n < NR) lds_read128<(n - 4) * 16 * RB>(Fb[BB ^ 1][n - 4], rb);
      else if constexpr (n < NR + ND) dma1(std::integral_constant<int, n - NR>{}, sbase, live, so);
    };
    static_for<0, 16>([&](auto mc) {
      // boustrophedon over the 4 x 4 fragment pairs: consecutive MFMAs share one operand register set
      constexpr int m = decltype(mc)::value, ib = m / 4, jb = (ib & 1) ? 3 - m % 4 : m % 4;
      acc[HALF * 4 + ib][jb] = Mma16<T>::run(__builtin_bit_cast(uint4, Fa[AB][ib]),
                                             __builtin_bit_cast(uint4, Fb[BB][jb]), acc[HALF * 4 + ib][jb]);
      if constexpr (m < 8) {   // two side operations behind each of the first eight MFMAs
        side(std::integral_constant<int, 2 * m>{});
        side(std::integral_constant<int, 2 * m + 1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I8 = std::integral_constant<int, LPS>;

  // prologue: fill the whole ring, wait for k-tile 0, fetch its first fragments
#pragma unroll
  for (int s = 0; s < NSTAGE; ++s) issue(s);
  wait_vmcnt<(NSTAGE - 1) * LPS>();
  __builtin_amdgcn_s_barrier();
  static_for<0, 4>([&](auto mc) {
    constexpr int m = decltype(mc)::value;
    lds_read128<m * 16 * RB>(Fa[0][m], offA[0]);
    lds_read128<m * 16 * RB>(Fb[0][m], offB[0]);
  });
  lds_wait8(Fa[0][0], Fa[0][1], Fa[0][2], Fa[0][3], Fb[0][0], Fb[0][1], Fb[0][2], Fb[0][3]);
  auto k_tile = [&](int64_t kt) {
    const uint32_t so_cur = (uint32_t)((kt % NSTAGE) * STAGE);
    phase(I0{}, I0{}, I0{}, I1{}, I0{}, I0{}, offA[0] + so_cur, 0u, 0);
    lds_wait4(Fa[1][0], Fa[1][1], Fa[1][2], Fa[1][3]);
    phase(I1{}, I0{}, I1{}, I0{}, I1{}, I0{}, offA[1] + so_cur, offB[1] + so_cur, 0);
    lds_wait8(Fa[0][0], Fa[0][1], Fa[0][2], Fa[0][3], Fb[1][0], Fb[1][1], Fb[1][2], Fb[1][3]);
    phase(I0{}, I1{}, I0{}, I1{}, I0{}, I0{}, offA[1] + so_cur, 0u, 0);
    lds_wait4(Fa[1][0], Fa[1][1], Fa[1][2], Fa[1][3]);
    // every fragment of k-tile kt is in registers: its slot can be refilled once all
    // waves are here, and k-tile kt+1 has landed once this wave's share of it has
    wait_vmcnt<(NSTAGE - 2) * LPS>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    const uint32_t so_next = (uint32_t)(((kt + 1) % NSTAGE) * STAGE);
    phase(I1{}, I1{}, I1{}, I0{}, I1{}, I8{}, offA[0] + so_next, offB[0] + so_next, kt + NSTAGE);
    lds_wait8(Fa[0][0], Fa[0][1], Fa[0][2], Fa[0][3], Fb[0][0], Fb[0][1], Fb[0][2], Fb[0][3]);
  };
  int64_t kt = 0;
  if constexpr (SYMK) {
    // first everything beyond the diagonal block, counted twice; then the block itself
    constexpr int64_t kDiagTiles = BO / BK_;
    const int64_t n_beyond = nk > kDiagTiles ? nk - kDiagTiles : 0;
    for (; kt < n_beyond; ++kt) k_tile(kt);
    if (n_beyond > 0) {
#pragma unroll
      for (int i = 0; i < IA; ++i)
#pragma unroll
        for (int j = 0; j < JB; ++j) acc[i][j] *= 2.0f;
    }
  }
  for (; kt < nk; ++kt) k_tile(kt);
  wait_vmcnt<0>();
  __syncthreads();

  // every LDS-DMA write has landed and every wave is past its last fragment read:
  // the tile memory is free for the per-token row sums and the Y_ref / output staging
  tile_epilogue<EPI, Acc16<IA, JB>, NWO, NWT, BT, (NSTAGE * STAGE >= NW * WO * WT * 2)>(
      a, acc, cand, to, tt, o0, t0, wo, wt, red, reinterpret_cast<float*>(lds));
#endif
}

// ---- host side ---------------------------------------------------------------
constexpr int kBO = 256, kBT = 256, kWO = 128, kWT = 64;
constexpr int64_t kChunkBytes = (int64_t)128 << 20;
constexpr int kDmaBK = 64, kDmaStages = 2;   // k-tile depth and LDS ring slots of the pipelined kernel
constexpr int kDmaThreads = 512;             // its 2 x 4 wave grid (128 x 64 outputs per wave)

void gemm_tile_counts(int64_t n_tok, int64_t c_out, int64_t* tiles_o, int64_t* tiles_t) {
  *tiles_o = ceil_div(c_out, kBO);
  *tiles_t = ceil_div(n_tok, kBT);
}

static GemmDev make_dev(const GemmArgs& g) {
  GemmDev d;
  d.X = (const uint16_t*)g.X; d.n_tok = g.n_tok; d.c_in = g.c_in; d.ldx = g.ldx;
  d.x_cand_stride = g.x_cand_stride; d.tok_scale = g.tok_scale;
  d.Wh = (const uint16_t*)g.Wh; d.c_out = g.c_out; d.ldw = g.ldw;
  d.w_cand_stride = g.w_cand_stride; d.n_cand = g.n_cand;
  d.Yref = g.Yref; d.ldy = g.ldy; d.ydt = g.yref_dtype; d.token_w = g.token_w;
  d.y_cand_stride = g.y_cand_stride; d.tri = g.tri ? 1 : 0;
  d.cand_outer = g.cand_outer ? 1 : 0; d.o_cand_stride = g.o_cand_stride;
  d.partial = g.partial; d.tok_partial = g.tok_partial;
  d.Yout = g.Yout; d.ldo = g.ldo; d.odt = g.yout_dtype;
  int64_t to, tt;
  gemm_tile_counts(g.n_tok, g.c_out, &to, &tt);
  d.tiles_o = (int)to; d.tiles_t = (int)tt;
  d.po = g.wide_patch ? 8 : 4; d.pt = PATCH_SLOTS / d.po;
  const int PATCH_O = d.po, PATCH_T = d.pt;
  d.npo = (int)ceil_div(to, PATCH_O); d.npt = (int)ceil_div(tt, PATCH_T);
  d.rag = (int)(to % PATCH_O);
  d.rag_pt = d.rag == 0 ? PATCH_T : PATCH_SLOTS / d.rag;   // e.g. 3 rows -> patches of 3 x 10
  // Tokens of one chunk.  While all tokens fit in half of the 256 MB last-level cache there is one
  // chunk.  Otherwise a chunk holds the largest power-of-two number of token patches within that
  // budget: with 1, 2, 4 or 8 patches per (candidate, patch row) the round-robin deal keeps every XCD
  // on the same token patch from one candidate to the next, which measured steadier (and on most
  // boxes faster) on 153,600-token inputs than 3, 5 or 6 patches, whose speed flips between
  // launches by up to 8 %.
  const int64_t patch_bytes = (int64_t)PATCH_T * kBT * g.c_in * 2;
  if ((int64_t)d.npt * patch_bytes <= kChunkBytes) {
    d.cpt = d.npt;
  } else {
    d.cpt = 1;
    while (d.cpt * 2 <= kXcd && (int64_t)d.cpt * 2 * patch_bytes <= kChunkBytes) d.cpt *= 2;
  }
  {
    const int n_full = d.rag ? d.npo - 1 : d.npo;
    const int64_t full_chunks = d.npt / d.cpt;
    const int cw_last = d.npt % d.cpt;
    auto per_cand = [&](int cw) {
      return (int64_t)n_full * cw + (d.rag ? (cw * PATCH_T + d.rag_pt - 1) / d.rag_pt : 0);
    };
    d.n_patches = (int64_t)g.n_cand * (full_chunks * per_cand(d.cpt) + (cw_last ? per_cand(cw_last) : 0));
  }
  return d;
}

// Whether launch_gemm_dot contracts only the upper part of a symmetric Wh (see SYMK).
// the pipelined kernel needs whole k-tiles and 32-bit byte offsets inside a 256-row panel
static bool pipelined_ok(const GemmArgs& g) {
  return (g.c_in % kDmaBK) == 0 && g.ldw < (1 << 21) && g.ldx < (1 << 21);
}
bool gemm_dot_symmetric(const GemmArgs& g) { return g.sym_k && g.c_out == g.c_in && pipelined_ok(g); }

template <int EPI>
static hipError_t launch_gemm(const GemmArgs& g, const char* name, hipStream_t stream) {
  GemmDev d = make_dev(g);
  const int64_t rounds = ceil_div(d.n_patches, kXcd);
  const int64_t blocks = rounds * kXcd * PATCH_SLOTS;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const bool dma = pipelined_ok(g);
  const bool symk = EPI == EPI_DOT && gemm_dot_symmetric(g);
  // (a symmetric product computes the tiles on and above the diagonal, a symmetric contraction
  // the k range from the diagonal block on: about half either way)
  const double tile_frac = (g.tri || symk) ? 0.5 * (1.0 + 1.0 / (double)d.tiles_o) : 1.0;
  ProfScope ps(name, stream, 2.0 * (double)g.n_tok * (double)g.c_in * (double)g.c_out * g.n_cand * tile_frac);
  constexpr int NT = (kBO / kWO) * (kBT / kWT) * 64;
  if (symk) {
    if constexpr (EPI == EPI_DOT) {
      if (!g.bf16)
        gemm_dma_kernel<F16, kDmaStages, EPI_DOT, true><<<(unsigned)blocks, kDmaThreads, 0, stream>>>(d);
      else
        gemm_dma_kernel<BF16, kDmaStages, EPI_DOT, true><<<(unsigned)blocks, kDmaThreads, 0, stream>>>(d);
    }
  } else if (dma) {
    if (!g.bf16)
      gemm_dma_kernel<F16, kDmaStages, EPI><<<(unsigned)blocks, kDmaThreads, 0, stream>>>(d);
    else
      gemm_dma_kernel<BF16, kDmaStages, EPI><<<(unsigned)blocks, kDmaThreads, 0, stream>>>(d);
  } else {
    if (!g.bf16) gemm_kernel<F16, kBO, kBT, kWO, kWT, EPI><<<(unsigned)blocks, NT, 0, stream>>>(d);
    else gemm_kernel<BF16, kBO, kBT, kWO, kWT, EPI><<<(unsigned)blocks, NT, 0, stream>>>(d);
  }
  return hipGetLastError();
}

// Host-side check of the block -> tile map for one problem shape, in both block orders (candidates
// inside every patch row, and candidate-outermost) and both patch shapes: walks every block id of the launch and counts
// how often each (candidate, tile) is produced.  Returns the number of tiles that are not produced
// exactly once (0 = both maps are bijections onto the tiles), or -1 for an invalid shape.
// *blocks_out receives the grid size.
int64_t tile_map_defects(int64_t n_tok, int64_t c_in, int64_t c_out, int n_cand, int64_t* blocks_out) {
  if (n_tok <= 0 || c_in <= 0 || c_out <= 0 || n_cand <= 0) return -1;
  int64_t bad = 0;
  for (int order = 0; order < 4; ++order) {
    GemmArgs g{};
    g.n_tok = n_tok; g.c_in = c_in; g.c_out = c_out; g.n_cand = n_cand;
    g.cand_outer = (order & 1) != 0; g.wide_patch = (order & 2) != 0;
    const GemmDev d = make_dev(g);
    const int64_t blocks = ceil_div(d.n_patches, kXcd) * kXcd * PATCH_SLOTS;
    if (blocks_out && order == 0) *blocks_out = blocks;
    const int64_t tiles = (int64_t)n_cand * d.tiles_o * d.tiles_t;
    unsigned char* seen = (unsigned char*)calloc((size_t)tiles, 1);
    if (!seen) return -1;
    for (int64_t b = 0; b < blocks; ++b) {
      int cand, to, tt;
      if (!decode_tile(d, b, cand, to, tt)) continue;
      if (cand < 0 || cand >= n_cand || to < 0 || tt < 0) { ++bad; continue; }
      unsigned char& c = seen[((int64_t)cand * d.tiles_o + to) * d.tiles_t + tt];
      if (c < 255) ++c;
    }
    for (int64_t i = 0; i < tiles; ++i) bad += seen[i] != 1;
    free(seen);
  }
  return bad;
}

hipError_t launch_gemm_loss(const GemmArgs& g, hipStream_t stream) {
  if (g.tok_partial) return launch_gemm<EPI_LOSS_TOK>(g, "gemm_loss_tok", stream);
  return launch_gemm<EPI_LOSS>(g, "gemm_loss", stream);
}
hipError_t launch_gemm_store(const GemmArgs& g, hipStream_t stream) {
  if (g.tri && g.n_tok != g.c_out) return hipErrorInvalidValue;
  if (g.n_cand != 1 && g.o_cand_stride == 0) return hipErrorInvalidValue;
  return launch_gemm<EPI_STORE>(g, g.tri ? "gemm_gram" : "gemm_store", stream);
}
hipError_t launch_gemm_dot(const GemmArgs& g, hipStream_t stream) {
  return launch_gemm<EPI_DOT>(g, "gemm_gram_loss", stream);
}

}  // namespace tlq
