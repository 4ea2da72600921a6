// Prefill side of Alg. 1 (Sec. III-C): gather every chunk into its bitwidth class
// (KV cache chunk reordering, Fig. 3), quantize + pack the INT2 / INT4 classes,
// copy the FP16 class.  One workgroup produces one 64-token block of the packed
// cache: 16-byte coalesced reads of the source rows, the block is assembled in LDS
// in its final layout and written out with 16-byte coalesced stores.
#include <hip/hip_runtime.h>

#include <cstring>

#include "common.h"
#include "exact_div.h"
#include "plan.h"

// The fp16 source is read once and the packed cache is written once: both bypass the caches
// (non-temporal), which leaves them to the kernels that run next.
#define RQ_LOAD(p) __builtin_nontemporal_load(p)
#define RQ_STORE(v, p) __builtin_nontemporal_store(v, p)

namespace cocktail {

struct RQParams {
  const void* plan;
  const RQItem* items;     // one record per block, in launch order
  const _Float16* src[2];  // K, V
  char* dst[2][kNumClasses];   // [K|V][class]
  int64_t stride_b, stride_h, stride_t;
  int32_t ragged;
  int32_t v_quads;         // V blocks in the token-quad form
  // paged source: token t of sequence b lives in page page_table[b * table_stride + t / page_size], slot t % page_size
  const int32_t* page_table;
  int64_t stride_page;
  int32_t page_size, table_stride, num_pages;
  int32_t page_shift;      // log2(page_size) if it is a power of two, else -1
  int32_t cls_first[kNumClasses];        // index of the first record of every class (prefix sums of class_blocks)
};

// min (or max) of v and a neighbour lane's v in one instruction: the neighbour's value arrives as a
// data-parallel-primitive operand.  The s_nop covers the wait states such an operand needs after the
// instruction that wrote it (the compiler cannot see into the asm).
#define COCKTAIL_DPP_MINMAX(NAME, OP, CTRL)                                                              \
  __device__ __forceinline__ float NAME(float v) {                                                     \
    float r;                                                                                           \
    asm("s_nop 1\n\t" OP " %0, %1, %1 " CTRL " row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));         \
    return r;                                                                                          \
  }
COCKTAIL_DPP_MINMAX(min_xor1, "v_min_f32_dpp", "quad_perm:[1,0,3,2]")
COCKTAIL_DPP_MINMAX(min_xor2, "v_min_f32_dpp", "quad_perm:[2,3,0,1]")
COCKTAIL_DPP_MINMAX(min_mirror8, "v_min_f32_dpp", "row_half_mirror")
COCKTAIL_DPP_MINMAX(min_mirror16, "v_min_f32_dpp", "row_mirror")
COCKTAIL_DPP_MINMAX(max_xor1, "v_max_f32_dpp", "quad_perm:[1,0,3,2]")
COCKTAIL_DPP_MINMAX(max_xor2, "v_max_f32_dpp", "quad_perm:[2,3,0,1]")
COCKTAIL_DPP_MINMAX(max_mirror8, "v_max_f32_dpp", "row_half_mirror")
COCKTAIL_DPP_MINMAX(max_mirror16, "v_max_f32_dpp", "row_mirror")
#undef COCKTAIL_DPP_MINMAX

// Minimum and maximum of the 8 fp16 channels in `raw`, then over the group of LPG = 4, 8 or 16 consecutive
// lanes (quad permutes, then mirrors of 8 and 16 lanes, whose quads are already uniform); every lane of the
// group ends up with both.  Packed fp16 min/max are exact; zeros of either sign compare equal, so a zero
// extreme is returned as +0 (x + 0 is x, and -0 + 0 is +0).
template <int LPG>
__device__ __forceinline__ void group_min_max(const u32x4& raw, float& mn, float& mx) {
  uint32_t lo01, lo23, hi01, hi23, lo, hi;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(lo01) : "v"(raw[0]), "v"(raw[1]));
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(lo23) : "v"(raw[2]), "v"(raw[3]));
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(hi01) : "v"(raw[0]), "v"(raw[1]));
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(hi23) : "v"(raw[2]), "v"(raw[3]));
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(lo) : "v"(lo01), "v"(lo23));
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(hi) : "v"(hi01), "v"(hi23));
  // low result half = min(low half, high half) of the pair
  asm("v_pk_min_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0]" : "=v"(lo) : "v"(lo));
  asm("v_pk_max_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0]" : "=v"(hi) : "v"(hi));
  mn = static_cast<float>(as_h2(lo).x);
  mx = static_cast<float>(as_h2(hi).x);
  mn = min_xor2(min_xor1(mn));
  mx = max_xor2(max_xor1(mx));
  if constexpr (LPG >= 8) mn = min_mirror8(mn), mx = max_mirror8(mx);
  if constexpr (LPG >= 16) mn = min_mirror16(mn), mx = max_mirror16(mx);
  mn += 0.0f;
  mx += 0.0f;
}

// f32(lo or hi half of w) - mn in one instruction: fma(f32(x), 1.0, -mn).  The conversion is exact and the
// fma rounds once, so this is the binary32 difference of the definition, bit for bit.
template <int HI>
__device__ __forceinline__ float half_minus(uint32_t w, float mn) {
  float d;
  if constexpr (HI) {
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(mn));
  } else {
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(mn));
  }
  return d;
}

// One token-group step of the quantizer on this lane's 8 channels (raw fp16 pairs).  Every operation
// gives the result of the single IEEE binary32 operation the definition asks for (x - mn: see half_minus;
// d * inv >= 0, so only the upper clamp can act).  The codes are returned as binary32 values, which are
// exact small integers: they are packed arithmetically (pack4) and converted once per half-word.
template <int BITS>
__device__ __forceinline__ void quantize8(const u32x4& raw, float mn, float mx, float (&code)[8], _Float16& scale_h) {
#pragma clang fp contract(off)
  constexpr float qmax = float((1 << BITS) - 1);
  const float r = mx - mn;
  const float s32 = div_by_qmax<(1 << BITS) - 1>(r);   // == r / qmax, bit for bit (exact_div.h)
  scale_h = static_cast<_Float16>(s32);
  const float sc = static_cast<float>(scale_h);
  // scale == 0 (a constant group, or a range that underflows fp16): all codes are 0.  No branch: the
  // differences are finite, and finite * 0 = 0.
  const float inv = sc == 0.0f ? 0.0f : recip_of_fp16_value(sc);   // == 1.0f / sc, bit for bit (exact_div.h)
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t w = raw[i >> 1];
    const float d = (i & 1) ? half_minus<1>(w, mn) : half_minus<0>(w, mn);
    code[i] = fminf(__builtin_rintf(d * inv), qmax);
  }
}

// a + b 2^BITS + c 2^(2 BITS) + d 2^(3 BITS) for codes held as binary32 integers: every intermediate is an
// integer below 2^16, so the fused multiply-adds are exact and replace the shifts and ors of a bit-field pack.
template <int BITS>
__device__ __forceinline__ float pack4(float a, float b, float c, float d) {
  constexpr float S = float(1 << BITS);
  return __builtin_fmaf(__builtin_fmaf(__builtin_fmaf(d, S, c), S, b), S, a);
}

// Quantizes this thread's rows (8 channels each; four rows at head_dim 128, two at head_dim 64) and writes codes
// and scale/zero pairs into the block image in shared memory (row form, or token quads for V where the cache
// stores V that way).
template <int D, int BITS, int G, class LoadRow>
__device__ __forceinline__ void quantize_rows(LoadRow load_row, char* lds, int row, int seg, bool quads,
                                              int meta_base) {
  constexpr int LPG = G / 8;   // lanes per group
  constexpr int NG = D / G;
  constexpr int RPP = 256 / (D / 8);    // rows per pass: the workgroup's 256 threads cover D / 8 lanes per row
  constexpr int PASSES = kTB / RPP;
  constexpr int PSTEP = RPP * 16;       // bytes between a thread's rows inside one 16-byte-piece plane
  const int qh = seg >> 3, qj = seg & 3, qe0 = 8 * ((seg >> 2) & 1);
  const bool writes_meta = (seg & (LPG - 1)) == 0;
  char* const meta0 = lds + meta_base + (row * NG + seg / LPG) * 4;
  // row form: INT8 has two words per lane, INT4 one; INT2 one word per lane pair, written by the even lane
  const int word = BITS == 8 ? 2 * seg : BITS == 4 ? seg : seg >> 1;
  char* const row0 = lds + ((word >> 2) * kTB + row) * 16 + (word & 3) * 4;
  // token quads: one half-word per 16 / BITS channels
  constexpr int QPH = BITS / 2;   // 16-byte pieces per 64-channel half of a row
  char* const quad0 = lds + quad_halfword_offset(QPH, 16 / BITS, row, qh, qj, qe0);
  char* const quad1 = lds + quad_halfword_offset(QPH, 16 / BITS, row, qh, qj, qe0 + (BITS == 8 ? 2 : 4));   // INT4: channels 4..7; INT8: 2, 3
  char* const quad2 = lds + quad_halfword_offset(QPH, 16 / BITS, row, qh, qj, qe0 + 4);   // INT8: channels 4, 5
  char* const quad3 = lds + quad_halfword_offset(QPH, 16 / BITS, row, qh, qj, qe0 + 6);   // INT8: channels 6, 7
#pragma unroll
  for (int pass = 0; pass < PASSES; ++pass) {
    const u32x4 raw = load_row(pass);
    float mn, mx;
    group_min_max<LPG>(raw, mn, mx);
    float c[8];
    _Float16 scale_h;
    quantize8<BITS>(raw, mn, mx, c, scale_h);
    if (writes_meta) {
      h2 m;
      m.x = scale_h;
      m.y = static_cast<_Float16>(mn);
      *reinterpret_cast<uint32_t*>(meta0 + pass * (RPP * NG * 4)) = as_u32(m);
    }
    if (quads) {
      // a half-word holds consecutive channels of one token, lowest channel in the lowest bits
      if constexpr (BITS == 8) {
        *reinterpret_cast<uint16_t*>(quad0 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(__builtin_fmaf(c[1], 256.0f, c[0])));
        *reinterpret_cast<uint16_t*>(quad1 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(__builtin_fmaf(c[3], 256.0f, c[2])));
        *reinterpret_cast<uint16_t*>(quad2 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(__builtin_fmaf(c[5], 256.0f, c[4])));
        *reinterpret_cast<uint16_t*>(quad3 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(__builtin_fmaf(c[7], 256.0f, c[6])));
      } else if constexpr (BITS == 4) {
        *reinterpret_cast<uint16_t*>(quad0 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(pack4<4>(c[0], c[1], c[2], c[3])));
        *reinterpret_cast<uint16_t*>(quad1 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(pack4<4>(c[4], c[5], c[6], c[7])));
      } else {
        const float lo = pack4<2>(c[0], c[1], c[2], c[3]), hi = pack4<2>(c[4], c[5], c[6], c[7]);
        *reinterpret_cast<uint16_t*>(quad0 + pass * PSTEP) = uint16_t(static_cast<uint32_t>(__builtin_fmaf(hi, 256.0f, lo)));
      }
    } else if constexpr (BITS == 8) {
      // row form, four channels per word: (c0, c2) in the low half-word, (c1, c3) in the high one
      u32x2 w;
      w.x = static_cast<uint32_t>(__builtin_fmaf(c[2], 256.0f, c[0])) | (static_cast<uint32_t>(__builtin_fmaf(c[3], 256.0f, c[1])) << 16);
      w.y = static_cast<uint32_t>(__builtin_fmaf(c[6], 256.0f, c[4])) | (static_cast<uint32_t>(__builtin_fmaf(c[7], 256.0f, c[5])) << 16);
      *reinterpret_cast<u32x2*>(row0 + pass * PSTEP) = w;
    } else {
      // row form: even channels in the low half-word, odd ones in the high half-word
      const uint32_t even = static_cast<uint32_t>(pack4<BITS>(c[0], c[2], c[4], c[6]));
      const uint32_t odd = static_cast<uint32_t>(pack4<BITS>(c[1], c[3], c[5], c[7]));
      const uint32_t mine = even | (odd << 16);
      if constexpr (BITS == 4) {
        *reinterpret_cast<uint32_t*>(row0 + pass * PSTEP) = mine;   // word = 8 channels
      } else {
        // word = 16 channels = two lanes: fields 0..3 of both half-words from the even lane, 4..7 from the odd one
        const uint32_t other = __shfl_xor(mine, 1);
        if ((seg & 1) == 0) *reinterpret_cast<uint32_t*>(row0 + pass * PSTEP) = mine | (other << 8);
      }
    }
  }
}

template <int D, int G, bool PAGED>
__global__ __launch_bounds__(256) void reorder_quantize_kernel(RQParams p) {
  static_assert(D == 64 || D == 128, "a row is 8 or 16 lanes of 8 channels");
  static_assert(D % G == 0, "a group lies inside a row");
  constexpr int SEGS = D / 8;           // lanes per row
  constexpr int RPP = 256 / SEGS;       // rows per pass
  constexpr int PASSES = kTB / RPP;
  __shared__ __attribute__((aligned(16))) char lds[kTB * 2 * D];

  const int which = blockIdx.y;  // 0 = K, 1 = V
  // everything about this block comes from one record; only blocks whose rows are not consecutive
  // source tokens (a chunk boundary or the tail inside the block) look the rows up one by one
  const RQItem item = load_record(p.items + blockIdx.x);
  const int cls = item.cls_nvalid & 0xff, nvalid = item.cls_nvalid >> 8;
  const int t0 = item.t0, j = item.j, b = item.b, h = item.h;
  const _Float16* src;       // row 0 of the block (consecutive rows) or token 0 of the head (row by row)
  bool per_row = t0 < 0;     // rows are looked up one by one
  if constexpr (PAGED) {
    src = p.src[which] + h * p.stride_h;     // the head inside a page; page and slot are added per block or per row
    const int last = t0 + (item.cls_nvalid >> 8) - 1;
    const int pg = t0 < 0 ? 0 : p.page_shift >= 0 ? t0 >> p.page_shift : t0 / p.page_size;
    if (t0 >= 0 && nvalid > 0 && (p.page_shift >= 0 ? last >> p.page_shift : last / p.page_size) == pg) {
      // the whole block lies inside one page: consecutive rows again
      const int page = p.page_table[int64_t(b) * p.table_stride + pg];
      if (uint32_t(page) < uint32_t(p.num_pages)) src += int64_t(page) * p.stride_page + int64_t(t0 - pg * p.page_size) * p.stride_t;
      else per_row = true;   // a page id outside the pool: the per-row path turns its rows into zeros
    } else {
      per_row = true;
    }
  } else if (p.ragged) {
    src = p.src[which] + item.ragged_row * p.stride_t;
  } else {
    src = p.src[which] + b * p.stride_b + h * p.stride_h + int64_t(t0 >= 0 ? t0 : 0) * p.stride_t;
  }
  const PlanHeader* hd = static_cast<const PlanHeader*>(p.plan);
  int C = 1, N = 0, cc0 = 0, chunk_tokens = 0;
  const int32_t* perm = nullptr;
  if (t0 < 0) {
    C = hd->chunk_size;
    const int32_t* chunk_off = plan_array<int32_t>(p.plan, hd->off_chunk_off);
    N = chunk_off[b + 1] - chunk_off[b];
    perm = plan_array<int32_t>(p.plan, hd->off_perm) + chunk_off[b];
    cc0 = plan_array<int32_t>(p.plan, hd->off_class_chunk0)[kNumClasses * b + cls];
    const int ntok = plan_array<int32_t>(p.plan, hd->off_class_tokens)[kNumClasses * b + cls];
    const int T = plan_array<int32_t>(p.plan, hd->off_seq_len)[b];
    chunk_tokens = (cls == kFp16Class) ? ntok - (T - N * C) : ntok;   // tokens of this class that come from chunks
  }

  const int tid = threadIdx.x;
  const int seg = tid % SEGS;      // 8 channels seg*8 .. seg*8+7
  const int row = tid / SEGS;      // this thread's rows of the block: row, row + RPP, ...
  const bool quads = which == 1 && p.v_quads != 0;   // token-quad form of V
  const int row_bytes = D * kClassBits[cls] / 8;

  // row `pass * 16 + row` of the block, 8 channels of it (zeros past the last valid row).  Consecutive
  // source rows (almost every block): one pointer per thread and a fixed step per pass.
  const _Float16* const row_ptr = src + int64_t(row) * p.stride_t + seg * 8;
  const int64_t pass_step = RPP * p.stride_t;
  // source token of row i of the block when the rows are looked up one by one
  auto token_of = [&](int i) {
    if (t0 >= 0) return t0 + i;
    const int r = j * kTB + i;      // row inside the class run of (b, h)
    if (r < chunk_tokens) {
      const int slot = r / C;
      return perm[cc0 + slot] * C + (r - slot * C);
    }
    return N * C + (r - chunk_tokens);   // Sec. III-A: tail tokens follow the FP16 chunks
  };
  // paged source, rows one by one: the page ids of this thread's four rows are fetched up front, so that
  // the four row loads do not each wait for a table look-up first (-1: not a page of the pool)
  int row_page[PASSES] = {};
  if constexpr (PAGED) {
    if (per_row) {
#pragma unroll
      for (int pass = 0; pass < PASSES; ++pass) {
        const int i = pass * RPP + row;
        int page = -1;
        if (i < nvalid) {
          const int t = token_of(i);
          page = p.page_table[int64_t(b) * p.table_stride + (p.page_shift >= 0 ? t >> p.page_shift : t / p.page_size)];
          if (uint32_t(page) >= uint32_t(p.num_pages)) page = -1;
        }
        row_page[pass] = page;
      }
    }
  }
  auto load_row = [&](int pass) {
    const int i = pass * RPP + row;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (i < nvalid) {
      const _Float16* ptr = row_ptr + pass * pass_step;
      if (per_row) {
        const int t = token_of(i);
        if constexpr (PAGED) {
          if (row_page[pass] < 0) return v;   // the row reads as zeros
          const int slot = p.page_shift >= 0 ? t & (p.page_size - 1) : t % p.page_size;
          ptr = src + int64_t(row_page[pass]) * p.stride_page + int64_t(slot) * p.stride_t + seg * 8;
        } else {
          ptr = src + int64_t(t) * p.stride_t + seg * 8;
        }
      }
      v = RQ_LOAD(reinterpret_cast<const u32x4*>(ptr));
    }
    return v;
  };

  // Where this thread's results go inside the block image in shared memory; every address is that of
  // row `row` plus a fixed step per pass (16 rows further: 256 bytes in every piece, 16 meta rows).
  // Token quads: the thread's channels are those of lane qj of a quad in the 64-channel half qh, its e-th
  // channels for e = qe0 .. qe0+7.
  const int qh = seg >> 3, qj = seg & 3, qe0 = 8 * ((seg >> 2) & 1);
  if (cls == kFp16Class) {
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
      const int i = pass * RPP + row;
      const u32x4 raw = load_row(pass);
      if (quads) {
#pragma unroll
        for (int x = 0; x < 8; ++x)
          *reinterpret_cast<uint16_t*>(lds + quad_halfword_offset(8, 1, i, qh, qj, qe0 + x)) =
              uint16_t((x & 1) ? raw[x >> 1] >> 16 : raw[x >> 1]);
      } else {
        *reinterpret_cast<u32x4*>(lds + (seg * kTB + i) * 16) = raw;
      }
    }
  } else if (cls == 0) {
    quantize_rows<D, 2, G>(load_row, lds, row, seg, quads, kTB * row_bytes);
  } else if (cls == 1) {
    quantize_rows<D, 4, G>(load_row, lds, row, seg, quads, kTB * row_bytes);
  } else {
    quantize_rows<D, 8, G>(load_row, lds, row, seg, quads, kTB * row_bytes);
  }
  __syncthreads();
  constexpr int NGc = D / G;
  const int bb = kTB * (row_bytes + (cls == kFp16Class ? 0 : 4 * NGc));
  char* dst = p.dst[which][cls] + int64_t(int(blockIdx.x) - p.cls_first[cls]) * bb;
  for (int o = tid * 16; o < bb; o += 256 * 16)
    RQ_STORE(*reinterpret_cast<const u32x4*>(lds + o), reinterpret_cast<u32x4*>(dst + o));
}

// Zeroes `n16` 16-byte words (the append buffers start out empty; rows that are never appended must
// read as finite values because the decode kernel loads whole 32-token units and masks afterwards).
__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* __restrict__ p, size_t n16) {
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += size_t(gridDim.x) * 256) p[i] = z;
}

// Exhaustive check of exact_div.h against the IEEE divisions, over every operand the quantizer can see.
__global__ __launch_bounds__(256) void selftest_div_kernel(unsigned long long* __restrict__ bad) {
  unsigned long long n3 = 0, n15 = 0, n255 = 0, nr = 0;
  const uint64_t stride = uint64_t(gridDim.x) * 256;
  // every non-negative float up to 131008 = 0x47FFE000
  for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x; i <= 0x47FFE000ull; i += stride) {
    const float r = __builtin_bit_cast(float, uint32_t(i));
    const float a3 = r / 3.0f, b3 = div_by_qmax<3>(r), a15 = r / 15.0f, b15 = div_by_qmax<15>(r);
    const float a255 = r / 255.0f, b255 = div_by_qmax<255>(r);
    n255 += __builtin_bit_cast(uint32_t, a255) != __builtin_bit_cast(uint32_t, b255) ||
            __builtin_bit_cast(uint16_t, static_cast<_Float16>(a255)) != __builtin_bit_cast(uint16_t, static_cast<_Float16>(b255));
    // the binary32 quotient and the fp16 scale made from it, as the quantizer makes it
    n3 += __builtin_bit_cast(uint32_t, a3) != __builtin_bit_cast(uint32_t, b3) ||
          __builtin_bit_cast(uint16_t, static_cast<_Float16>(a3)) != __builtin_bit_cast(uint16_t, static_cast<_Float16>(b3));
    n15 += __builtin_bit_cast(uint32_t, a15) != __builtin_bit_cast(uint32_t, b15) ||
           __builtin_bit_cast(uint16_t, static_cast<_Float16>(a15)) != __builtin_bit_cast(uint16_t, static_cast<_Float16>(b15));
  }
  // every positive finite fp16 value
  for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x + 1; i < 0x7C00u; i += stride) {
    const float x = static_cast<float>(__builtin_bit_cast(_Float16, uint16_t(i)));
    nr += __builtin_bit_cast(uint32_t, 1.0f / x) != __builtin_bit_cast(uint32_t, recip_of_fp16_value(x));
  }
  if (n3) atomicAdd(bad + 0, n3);
  if (n15) atomicAdd(bad + 1, n15);
  if (nr) atomicAdd(bad + 2, nr);
  if (n255) atomicAdd(bad + 3, n255);
}

}  // namespace cocktail

using namespace cocktail;

extern "C" int cocktail_selftest_arithmetic(uint64_t* mismatches, void* stream) {
  if (!mismatches) return fail(COCKTAIL_EINVAL, "mismatches is NULL");
  if (reinterpret_cast<uintptr_t>(mismatches) & 7) return fail(COCKTAIL_EALIGN, "mismatches must be 8-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<u32x4*>(mismatches), size_t(2));
  hipLaunchKernelGGL(selftest_div_kernel, dim3(4096), dim3(256), 0, st,
                     reinterpret_cast<unsigned long long*>(mismatches));
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "selftest launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}


namespace {

// Checks the cache against its plan, fills the destination part of the parameters and launches: the append
// buffers are cleared, then one launch covers K and V of all classes.
int launch_reorder_quantize(const cocktail_shape* shape, const cocktail_cache* cache, const PlanHeader* hd, RQParams p,
                            bool paged, void* stream) {
  if (reinterpret_cast<uintptr_t>(cache->plan_dev) & 15) return fail(COCKTAIL_EALIGN, "plan_dev must be 16-byte aligned");
  p.plan = cache->plan_dev;
  p.items = reinterpret_cast<const RQItem*>(static_cast<const char*>(cache->plan_dev) + hd->off_rq_items);
  int64_t tot = 0;
  for (int c = 0; c < kNumClasses; ++c) {
    if (hd->class_bytes[c] > 0 && (!cache->k[c] || !cache->v[c]))
      return fail(COCKTAIL_EINVAL, "cache buffer of class %d is NULL but %lld bytes are needed", c,
                  (long long)hd->class_bytes[c]);
    if ((reinterpret_cast<uintptr_t>(cache->k[c]) | reinterpret_cast<uintptr_t>(cache->v[c])) & 15)
      return fail(COCKTAIL_EALIGN, "cache buffers must be 16-byte aligned");
    p.dst[0][c] = static_cast<char*>(cache->k[c]);
    p.dst[1][c] = static_cast<char*>(cache->v[c]);
    p.cls_first[c] = static_cast<int32_t>(tot);
    tot += hd->class_blocks[c];
  }
  if (tot >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "too many blocks for one launch");
  p.v_quads = hd->v_layout;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hd->append_capacity > 0) {
    if (!cache->k_app || !cache->v_app) return fail(COCKTAIL_EINVAL, "the plan has append buffers but k_app or v_app is NULL");
    if ((reinterpret_cast<uintptr_t>(cache->k_app) | reinterpret_cast<uintptr_t>(cache->v_app)) & 15)
      return fail(COCKTAIL_EALIGN, "append buffers must be 16-byte aligned");
    const size_t n16 = size_t(hd->batch) * hd->num_kv_heads * hd->append_blocks * (kTB * 2 * shape->head_dim / 16);
    const unsigned blocks = static_cast<unsigned>(n16 / 256 < 4096 ? (n16 + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, static_cast<u32x4*>(cache->k_app), n16);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, static_cast<u32x4*>(cache->v_app), n16);
  }
  if (tot == 0) return COCKTAIL_OK;
  const dim3 grid(static_cast<unsigned>(tot), 2, 1), block(256, 1, 1);
#define COCKTAIL_RQ_LAUNCH(D, G)                                                                 \
  if (paged) hipLaunchKernelGGL((reorder_quantize_kernel<D, G, true>), grid, block, 0, st, p);  \
  else hipLaunchKernelGGL((reorder_quantize_kernel<D, G, false>), grid, block, 0, st, p)
  if (shape->head_dim == 64) {
    if (shape->group_size == 32) COCKTAIL_RQ_LAUNCH(64, 32);
    else COCKTAIL_RQ_LAUNCH(64, 64);
  } else {
    switch (shape->group_size) {
      case 32: COCKTAIL_RQ_LAUNCH(128, 32); break;
      case 64: COCKTAIL_RQ_LAUNCH(128, 64); break;
      default: COCKTAIL_RQ_LAUNCH(128, 128); break;
    }
  }
#undef COCKTAIL_RQ_LAUNCH
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "reorder_quantize launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}

int plan_of(const cocktail_shape* shape, const cocktail_cache* cache, const PlanHeader** out) {
  if (int rc = check_shape(shape)) return rc;
  if (!cache || !cache->plan_host || !cache->plan_dev) return fail(COCKTAIL_EINVAL, "cache or its plan is NULL");
  const PlanHeader* hd = static_cast<const PlanHeader*>(cache->plan_host);
  if (hd->magic != kPlanMagic || hd->version != kPlanVersion)
    return fail(COCKTAIL_EINVAL, "plan_host is not a plan written by this library version");
  if (hd->batch != shape->batch || hd->num_kv_heads != shape->num_kv_heads || hd->head_dim != shape->head_dim ||
      hd->chunk_size != shape->chunk_size || hd->group_size != shape->group_size ||
      hd->num_q_heads != shape->num_q_heads)
    return fail(COCKTAIL_EINVAL, "plan was made for a different shape");
  if (shape->head_dim != 64 && shape->head_dim != 128)
    return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 64 and 128, got %d", shape->head_dim);
  *out = hd;
  return COCKTAIL_OK;
}

}  // namespace

extern "C" int cocktail_reorder_quantize(const cocktail_shape* shape, const void* k_src, const void* v_src,
                                         int32_t src_layout, int64_t stride_b, int64_t stride_h,
                                         int64_t stride_t, const cocktail_cache* cache, void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = plan_of(shape, cache, &hd)) return rc;
  if (src_layout != COCKTAIL_SRC_STRIDED && src_layout != COCKTAIL_SRC_RAGGED)
    return fail(COCKTAIL_EINVAL, "unknown src_layout %d (a paged source goes through cocktail_reorder_quantize_paged)", src_layout);
  if (hd->total_tokens > 0 && (!k_src || !v_src)) return fail(COCKTAIL_EINVAL, "k_src or v_src is NULL");
  if ((reinterpret_cast<uintptr_t>(k_src) | reinterpret_cast<uintptr_t>(v_src) |
       reinterpret_cast<uintptr_t>(cache->plan_dev)) & 15)
    return fail(COCKTAIL_EALIGN, "k_src, v_src and plan_dev must be 16-byte aligned");
  if (stride_t < shape->head_dim || (stride_t & 7))
    return fail(COCKTAIL_EINVAL, "stride_t %lld must be >= head_dim and a multiple of 8", (long long)stride_t);
  if (src_layout == COCKTAIL_SRC_STRIDED && (stride_b < 0 || stride_h < 0 || (stride_b & 7) || (stride_h & 7)))
    return fail(COCKTAIL_EINVAL, "stride_b and stride_h must be non-negative multiples of 8");
  RQParams p;
  std::memset(&p, 0, sizeof(p));
  p.src[0] = static_cast<const _Float16*>(k_src);
  p.src[1] = static_cast<const _Float16*>(v_src);
  p.stride_b = stride_b, p.stride_h = stride_h, p.stride_t = stride_t;
  p.ragged = (src_layout == COCKTAIL_SRC_RAGGED);
  return launch_reorder_quantize(shape, cache, hd, p, false, stream);
}

extern "C" int cocktail_reorder_quantize_paged(const cocktail_shape* shape, const cocktail_paged_source* src,
                                               const cocktail_cache* cache, void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = plan_of(shape, cache, &hd)) return rc;
  if (!src) return fail(COCKTAIL_EINVAL, "src is NULL");
  if (src->reserved != 0) return fail(COCKTAIL_EINVAL, "cocktail_paged_source::reserved must be zero");
  if (src->page_size < 1 || src->num_pages < 1 || src->table_stride < 0)
    return fail(COCKTAIL_EINVAL, "page_size and num_pages must be >= 1, table_stride >= 0");
  if (hd->total_tokens > 0 && (!src->k_pages || !src->v_pages || !src->page_table))
    return fail(COCKTAIL_EINVAL, "k_pages, v_pages or page_table is NULL");
  if ((reinterpret_cast<uintptr_t>(src->k_pages) | reinterpret_cast<uintptr_t>(src->v_pages)) & 15)
    return fail(COCKTAIL_EALIGN, "k_pages and v_pages must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(src->page_table) & 3) return fail(COCKTAIL_EALIGN, "page_table must be 4-byte aligned");
  if (src->stride_t < shape->head_dim || (src->stride_t & 7))
    return fail(COCKTAIL_EINVAL, "stride_t %lld must be >= head_dim and a multiple of 8", (long long)src->stride_t);
  if (src->stride_page < 0 || src->stride_h < 0 || (src->stride_page & 7) || (src->stride_h & 7))
    return fail(COCKTAIL_EINVAL, "stride_page and stride_h must be non-negative multiples of 8");
  const int32_t* seq_len = plan_array<int32_t>(cache->plan_host, hd->off_seq_len);
  for (int b = 0; b < hd->batch; ++b) {
    const int64_t need = (int64_t(seq_len[b]) + src->page_size - 1) / src->page_size;
    if (need > src->table_stride)
      return fail(COCKTAIL_EINVAL, "sequence %d has %d tokens = %lld pages of %d, but a page table row holds %d entries",
                  b, seq_len[b], (long long)need, src->page_size, src->table_stride);
  }
  RQParams p;
  std::memset(&p, 0, sizeof(p));
  p.src[0] = static_cast<const _Float16*>(src->k_pages);
  p.src[1] = static_cast<const _Float16*>(src->v_pages);
  p.stride_h = src->stride_h, p.stride_t = src->stride_t, p.stride_page = src->stride_page;
  p.page_table = src->page_table;
  p.page_size = src->page_size, p.table_stride = src->table_stride, p.num_pages = src->num_pages;
  p.page_shift = -1;
  for (int sft = 0; sft < 31; ++sft)
    if (src->page_size == (1 << sft)) p.page_shift = sft;
  return launch_reorder_quantize(shape, cache, hd, p, true, stream);
}
