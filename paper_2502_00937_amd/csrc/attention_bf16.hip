// Variable-length flash attention on bf16 MFMA.  A work item is a block of 128 query rows of
// one segment (a tile, or all tiles of an image); keys never come from outside the segment, so
// no padding or masking crosses images.
//
// Everything is computed transposed so that a lane owns one query for the whole kernel:
//   S^T[key, q]  = K[key, :] . Q[q, :]       (A = K tile from LDS, B = Q^T held in registers)
//   O^T[d, q]   += V^T[d, key] . P^T[key, q] (A = V^T fragments, taken from the V tile in LDS with the
//                                             transposing read; B = P^T straight from the S^T
//                                             accumulator registers)
// With the 32x32 MFMA accumulator layout (lane = column q, registers = rows) the softmax
// statistics of a query are per-lane scalars, the row maximum needs one exchange with lane^32,
// and the P^T operand of the second product is the accumulator of the first, converted in
// place: registers 8s..8s+7 of an S^T block are exactly the 8 k-values lane group g feeds
// to k-step s, provided V^T is read in the same key order (keys 16s + 8jj + 4g + i).
//
// The vector instructions of one wave do overlap the MFMAs of another wave on the same SIMD (a probe: a wave
// issuing only MFMAs keeps its 32 clocks per instruction while a second wave on the SIMD issues fma or exp2
// back to back and is slowed by about 12 %), so the kernel is shaped around the number of waves per SIMD and the
// vector instruction count per 32 x 32 block of logits: a wave owns 32 queries, which keeps it at 128-168 VGPRs
// so that four (head dim 64) or three waves from different workgroups share a SIMD and interleave their
// dependency chains (a fourth wave is worth 7 % at head dim 64); the queries arrive multiplied by
// log2(e) / sqrt(head dim), so the logits are exp2 arguments as they leave the first product; full key tiles
// carry no mask code at all (a segment's last tile is a separate instantiation that also skips an empty key
// half, and waves with no valid query row skip the arithmetic); and the normal pass uses no reference maximum:
// see `attend` below.
// K/V tiles of 64 keys are double-buffered in LDS: the next tile's global loads are issued before
// the current tile is processed and written to the other buffer afterwards (one barrier per tile).
// Both tiles are stored as they are loaded, whole rows of 16-byte pieces; ds_read_b64_tr_b16 hands the
// second product its V^T fragments (four keys of one column per lane and instruction).  A V tile
// transposed on its way into LDS (v_perm_b32 and eight 4-byte stores per 16-byte piece, loads of 16
// bytes from 32 different rows per instruction) cost the kernel 4 % at head dim 64 and 10 % at 72.
#include <type_traits>

#include "common.h"

namespace vitenc {

namespace {

constexpr int AKV = 64;  // keys per LDS tile
enum { SUM_VALU = 0, SUM_ROWS = 1 };
constexpr float REFERENCE_LIMIT = 18446744073709551616.0f;  // 2^64: a row sum this large moves the reference maximum

// QB = 32-query blocks per wave, NW = waves per workgroup: a work item is 32 * QB * NW query rows.
// All head dims run QB = 1, NW = 4 (128 rows); QB = 2 (each K / V^T fragment feeding two MFMAs, two
// waves per SIMD) was measured 15 % slower.
// DHP = head dim as stored (a multiple of 8: 64, 72, 80, 96, 128).  The S^T product runs over DHL = DHP rounded up
// to whole 16-wide k-steps: for 72 the K tile's LDS rows carry 8 zero columns (written once, never by the loader)
// and the Q fragment of the last half k-step is zero, so nothing is padded in HBM.
template <int DHP, int QB, int NW>
struct AttnShape {
  static constexpr int DHL = (DHP + 15) / 16 * 16;  // head dim of the K rows in LDS
  static constexpr int ANT = 64 * NW;            // threads per workgroup
  static constexpr int AQ = 32 * QB * NW;        // query rows per work item
  static constexpr int KS = DHL / 16;            // k-steps of the S^T product
  static constexpr int DB = (DHP + 31) / 32;     // 32-row blocks of O^T
  static constexpr int NCH = DHP / 8;            // 16-byte chunks per K/V row
  static constexpr int K_STRIDE = DHL * 2 + 16;  // bytes per K row in LDS (padding kills bank conflicts)
  // V rows in LDS: the head dim, then the spare rows of the last O^T block as extra columns (zeros, or ones for the
  // row sums, see SUM).  The second product's V^T fragments are read with the transposing LDS read; half a wave
  // fetches 4 keys x 64 bytes at a time, which fall on the 64 banks once each when the row stride is 64 bytes
  // times an odd number (192 bytes for the head dims with 96 columns, 320 for 128).  Head dim 64 would need 192
  // bytes for its 128, and four workgroups would no longer fit a unit's LDS: its rows are 128 bytes with no padding,
  // and the rows of every second pair of keys keep their two 64-byte halves swapped (V_SWAP), which does the same.
  static constexpr int V_COLS = DB * 32;
  static constexpr bool V_SWAP = DHP == 64;
  static constexpr int V_STRIDE = V_SWAP ? 128 : ((V_COLS * 2 + 63) / 64 | 1) * 64;
  static constexpr int K_BYTES = AKV * K_STRIDE;
  static constexpr int V_BYTES = AKV * V_STRIDE;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int K_ITEMS = AKV * NCH;  // 16-byte chunks of the K tile, and of the V tile
  static constexpr int K_PER = (K_ITEMS + ANT - 1) / ANT;
  // where the row sums of P come from in the fast pass: spare rows of the last O^T block if the head dim leaves
  // any (72, 80: two columns of ones in the V rows' padding), vector instructions otherwise (v_dot2c_f32_bf16 of a packed pair with a pair of ones: 8 per
  // block of logits).  (One more accumulator fed by a fragment of ones held in registers costs 20 registers: at
  // head dim 64 that is the fourth wave of a SIMD, and the kernel came out 5 % slower with it, 13 % when forced
  // into 128 registers.)
  static constexpr int SUM = DB * 32 - DHP >= 8 ? SUM_ROWS : SUM_VALU;
};

template <int DHP, int QB, int NW>
__global__ __launch_bounds__(64 * NW, QB == 1 ? (DHP == 64 ? 4 : DHP <= 96 ? 3 : 2) : 2) void attention_bf16_kernel(const AttnArgs a) {
  using Sh = AttnShape<DHP, QB, NW>;
  constexpr int ANT = Sh::ANT;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // 2 stages of (K tile, V tile)

  // Workgroup ids are dealt round-robin to the 8 XCDs.  Consecutive work items are the query
  // blocks of one segment, which read the same K and V rows: give each XCD a contiguous run of
  // work items so those rows are fetched into one L2 only.
  const int per_xcd = (a.n_work + 7) >> 3;
  const int wi = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (wi >= a.n_work) return;
  const AttnWork w = a.work[a.reverse ? a.n_work - 1 - wi : wi];
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, g = lane >> 5;
  const int partner_addr = (lane ^ 32) << 2;  // ds_bpermute byte address of the lane that holds the other 16 keys of a query
  // The transposing LDS read (ds_read_b64_tr_b16) works on groups of 16 lanes: lane j of a group points at 8 bytes
  // (four 16-bit values), and lane i receives value i % 4 of the lanes i / 4, i / 4 + 4, i / 4 + 8 and i / 4 + 12.
  // A lane (lq, g) of the second product needs V[key0 + 4 g + e][32 b + lq], e = 0 .. 3: with lane j of group G
  // (lq = 16 (G % 2) + i, g = G / 2) pointing at V[key0 + 4 g + j / 4][32 b + 16 (G % 2) + 4 (j % 4) .. + 3], the
  // lanes j = i / 4 + 4 e hold exactly the keys key0 + 4 g + e at the four columns that contain this lane's.
  // (V_SWAP: the lane's key is key0 + 4 g + j / 4 with key0 a multiple of 8, so bit 1 of the key is bit 3 of j, and
  //  the swap turns column block b into b ^ 1 for those lanes)
  const uint32_t vt_off = (uint32_t)((4 * (lane >> 5) + ((lane & 15) >> 2)) * Sh::V_STRIDE + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);
  const uint32_t vt_swap = Sh::V_SWAP && (lane & 8) ? 64u : 0u;
  auto read_tr = [](const unsigned char* q) {
    typedef short v4s __attribute__((ext_vector_type(4)));
    const v4s v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)q);
    return __builtin_bit_cast(u32x2, v);
  };
  // this head's Q, K and V: column blocks of the [rows, ld_qkv] matrix, or (qkv_rows != 0) blocks of their own,
  // [qkv_rows, DHP] each with consecutive rows.  Either way: a base and a row stride.
  const size_t blk = a.qkv_rows ? a.qkv_rows * DHP : (size_t)DHP;  // elements from one head's block to the next
  const int row_elems = a.qkv_rows ? DHP : a.ld_qkv;
  const bf16_t* q_base = (const bf16_t*)a.qkv + (size_t)head * blk;
  const bf16_t* k_base = (const bf16_t*)a.qkv + (size_t)(a.heads + head) * blk;
  const bf16_t* v_base = (const bf16_t*)a.qkv + (size_t)(2 * a.heads + head) * blk;
  const int seg_end = w.seg_start + w.seg_len;

  // Q^T fragments of the wave's two query blocks: lane holds d = 16*ks + 8*g .. +8 of its query row;
  // rows past the segment end compute on a copy of its last row and are never stored.
  bf16x8 qf[QB][Sh::KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qload = min(w.q0 + (wave * QB + qb) * 32 + lq, seg_end - 1);
#pragma unroll
    for (int ks = 0; ks < Sh::KS; ++ks) {
      if (ks * 16 + 8 < DHP) {  // both 8-wide halves of the k-step lie inside the head
        qf[qb][ks] = *(const bf16x8*)(q_base + (size_t)qload * row_elems + ks * 16 + g * 8);
      } else {  // head dim 72: the upper half of the last k-step does not exist; its lanes feed zeros
        const bf16x8 lo = *(const bf16x8*)(q_base + (size_t)qload * row_elems + ks * 16);
        const u32x4 z = {0u, 0u, 0u, 0u};
        qf[qb][ks] = g == 0 ? lo : __builtin_bit_cast(bf16x8, z);
      }
    }
  }

  u32x4 rk[Sh::K_PER], rv[Sh::K_PER];
  // global -> registers.  Each thread's (row, column) inside a tile is fixed, so its byte offsets
  // are computed once; only a segment's last tile clamps rows past the end to the last row (their
  // logits are masked, the clamped values only need to be finite).
  const uint32_t row_bytes = (uint32_t)row_elems * 2u;
  const unsigned char* seg_k = (const unsigned char*)(k_base + (size_t)w.seg_start * row_elems);
  const unsigned char* seg_v = (const unsigned char*)(v_base + (size_t)w.seg_start * row_elems);
  // Each thread's (row, column) inside a tile is fixed: its byte offsets from the tile's first row are
  // computed once, and a full tile is loaded from a wave-uniform base plus those offsets with no
  // address arithmetic at all.  Only a segment's last, partial tile clamps rows past the end to the
  // last row (their logits are masked, the clamped values only need to be finite).
  uint32_t k_off[Sh::K_PER];  // (V rows are read at the same offsets from their own base)
#pragma unroll
  // (threads whose item index lies past the tile's last item load the last item again and do not
  //  store it: no load sits under divergent control flow)
  for (int i = 0; i < Sh::K_PER; ++i) {
    const int it = min(tid + i * ANT, Sh::K_ITEMS - 1), key = it / Sh::NCH;
    k_off[i] = (uint32_t)key * row_bytes + (uint32_t)((it - key * Sh::NCH) * 8) * 2u;
  }
  auto load_tile = [&](int k0, auto partial_tag) {
    constexpr bool PARTIAL = decltype(partial_tag)::value;
    const unsigned char* tile_k = seg_k + (size_t)k0 * row_bytes;  // wave-uniform
    const unsigned char* tile_v = seg_v + (size_t)k0 * row_bytes;
    const int last = w.seg_len - 1 - k0;  // largest valid row index inside this tile (>= 0)
#pragma unroll
    for (int i = 0; i < Sh::K_PER; ++i) {
      const int it = min(tid + i * ANT, Sh::K_ITEMS - 1);
      uint32_t off = k_off[i];
      if (PARTIAL) {
        const int key = it / Sh::NCH;
        off -= (uint32_t)(key - min(key, last)) * row_bytes;
      }
      rk[i] = *(const u32x4*)(tile_k + off);
      rv[i] = *(const u32x4*)(tile_v + off);
    }
  };
  // registers -> LDS, K and V rows alike (the second product reads V through the transposing LDS read)
  auto store_tile = [&](unsigned char* sK, unsigned char* sV) {
#pragma unroll
    for (int i = 0; i < Sh::K_PER; ++i) {
      const int it = tid + i * ANT;
      if (Sh::K_ITEMS % ANT == 0 || it < Sh::K_ITEMS) {
        const int key = it / Sh::NCH, ch = it - key * Sh::NCH;
        *(u32x4*)(sK + key * Sh::K_STRIDE + ch * 16) = rk[i];
        *(u32x4*)(sV + key * Sh::V_STRIDE + (Sh::V_SWAP && (key & 2) ? ch ^ 4 : ch) * 16) = rv[i];
      }
    }
  };

  const int n_tiles = (w.seg_len + AKV - 1) / AKV;
  // a wave whose 32 * QB query rows all lie past the segment end (last block of a segment) skips the arithmetic
  const bool wave_active = w.q0 + wave * QB * 32 < seg_end;

  // What the loader never writes must still be finite (a product with garbage could be NaN): the K rows' columns
  // DHP .. DHL - 1 take part in S^T and are zero.  The V rows' columns DHP .. 32 DB - 1 only produce O^T rows that are
  // never stored; they are zero, except that with SUM_ROWS two of them hold ones, so that the row sums of P come
  // out of the second product for nothing (column DHP for the lanes with g = 0, column DHP + 4 for those with
  // g = 1: the same accumulator register).  Both stages, once.
  if constexpr (Sh::DHL > DHP || Sh::DB * 32 > DHP) {
#pragma unroll
    for (int stg = 0; stg < 2; ++stg) {
      unsigned char* sK = lds + stg * Sh::STAGE;
      unsigned char* sV = sK + Sh::K_BYTES;
      if constexpr (Sh::DHL > DHP) {
        static_assert(Sh::DHL - DHP == 8 || Sh::DHL == DHP, "at most one 16-byte chunk of padding per K row");
        for (int key = tid; key < AKV; key += ANT) *(u32x4*)(sK + key * Sh::K_STRIDE + DHP * 2) = u32x4{0u, 0u, 0u, 0u};
      }
      constexpr int PAD_WORDS = (Sh::V_COLS - DHP) / 2;  // 4-byte words of padding per V row
      for (int it = tid; it < AKV * PAD_WORDS; it += ANT) {
        const int key = it / PAD_WORDS, wd = it % PAD_WORDS;  // word wd holds columns DHP + 2 wd and DHP + 2 wd + 1
        const uint32_t fill = Sh::SUM == SUM_ROWS && (wd == 0 || wd == 2) ? 0x00003F80u : 0u;  // a bf16 one, a zero
        *(uint32_t*)(sV + key * Sh::V_STRIDE + DHP * 2 + wd * 4) = fill;
      }
    }
  }

  f32x16 o[QB][Sh::DB];
  float l[QB];  // row sums of P (FAST with SUM_VALU, and the general pass)
  float m[QB];  // reference maximum in log2 units (general pass)

  // One pass over the segment's K/V tiles.
  //
  // FAST (the pass that normally is the only one): P^T = exp2(S^T) with no reference maximum at all.  The logits
  // arrive in log2 units (the QKV product has multiplied the queries by log2(e) / sqrt(head dim)), P is a bf16
  // value and the sums are fp32, eight exponent bits both, so nothing is lost while the row sum stays between
  // 2^-100 and 2^100, i.e. while the largest logit of a row lies within about +-69 (natural units) of zero.  That
  // is checked once, after the last tile; a workgroup with a row outside runs the general pass instead.  Per
  // 32 x 32 block of logits this pass issues 16 exp2, 8 packed conversions and its MFMAs; the row sums come from
  // the matrix cores where the head dim leaves spare rows in the last O^T block (SUM_ROWS: two columns of ones in the
  // V tile's padding), else from 8 two-element dot products with ones (SUM_VALU).  Either way the sum is taken
  // over the rounded weights, the ones the second product multiplies with.
  //
  // General pass: the online softmax with a lazily moving reference maximum m.  m only has to keep exp2 in range,
  // not to be the exact running maximum, so the row maximum is not computed on its common path either: a row sum
  // that reaches 2^64 (or is not a number: m = -inf before the first tile) says that m has to move; only then is
  // the maximum of the half tile taken, m moved and the accumulators rescaled.
  auto attend = [&](auto fast_tag) {
    constexpr bool FAST = decltype(fast_tag)::value;
    constexpr int SUM = FAST ? Sh::SUM : SUM_VALU;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[qb][b][v] = 0.f;
      m[qb] = -INFINITY;
      l[qb] = 0.f;
    }
    if (w.seg_len >= AKV) load_tile(0, std::false_type{});
    else load_tile(0, std::true_type{});
    store_tile(lds, lds + Sh::K_BYTES);
    __syncthreads();

    // One K/V tile.  MASK is set only for a segment's last, partial tile: full tiles carry no
    // per-logit compare/select at all.
    auto process_tile = [&](int t, auto mask_tag) {
      constexpr bool MASK = decltype(mask_tag)::value;
      const unsigned char* sK = lds + (t & 1) * Sh::STAGE;
      const unsigned char* sV = sK + Sh::K_BYTES;
      if (t + 1 < n_tiles) {  // the next tile is full unless it is the segment's last, partial one
        if ((t + 2) * AKV <= w.seg_len) load_tile((t + 1) * AKV, std::false_type{});
        else load_tile((t + 1) * AKV, std::true_type{});
      }

      const int remaining = w.seg_len - t * AKV;  // valid keys in this tile (may exceed AKV)
      // the tile is processed in two 32-key halves to keep S^T and P^T small in registers
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        if (!wave_active) break;  // (the wave still stages K / V and meets the barriers)
        if (MASK && kb * 32 >= remaining) break;  // the second half of the last tile may hold no key at all
        // ---- S^T = K . Q^T: each K fragment feeds all query blocks of the wave; keys past the segment end are
        //      masked (only a segment's last tile has any)
        f32x16 st[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int v = 0; v < 16; ++v) st[qb][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < Sh::KS; ++ks) {
          const bf16x8 kf = *(const bf16x8*)(sK + (kb * 32 + lq) * Sh::K_STRIDE + (ks * 2 + g) * 16);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            st[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][ks], st[qb], 0, 0, 0);
        }
        if (MASK) {
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = kb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
              if (key >= remaining) st[qb][v] = -INFINITY;
            }
        }
        // ---- P^T replaces S^T as bf16 fragments
        bf16x8 pf[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          float psum;
          auto exponentials = [&](const f32x16& sq, float neg_m) {
            psum = 0.f;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
              float p[8];
#pragma unroll
              for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(FAST ? sq[s2 * 8 + e] : sq[s2 * 8 + e] + neg_m);
              const uint32_t pw[4] = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]),
                                      pack_bf16x2(p[6], p[7])};
              const u32x4 pk = {pw[0], pw[1], pw[2], pw[3]};
              if (SUM == SUM_VALU) {
                // the row sum is taken over the rounded weights, the ones the second product multiplies with, two
                // per instruction: v_dot2c_f32_bf16 with a pair of ones (fp32 accumulation).  (The packed words are
                // taken from the scalar array: cast from the elements of the vector `pk`, this compiler gave all
                // four instructions the vector's first register.)
                const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[e]), ones, psum, false);
              }
              pf[qb][s2] = __builtin_bit_cast(bf16x8, pk);
            }
          };
          exponentials(st[qb], -m[qb]);
          if constexpr (!FAST) {
            if (__builtin_amdgcn_ballot_w64(!(psum < REFERENCE_LIMIT)) != 0) {
              // Rare: move m to the maximum seen so far (the same for the two lanes that share a query), rescale
              // the accumulators and redo the exponentials.  (Forming the logits again here instead of keeping
              // them alive costs head dims 80 and 96 seven per cent: measured.)
              const f32x16& sr = st[qb];
              float mx = sr[0];
#pragma unroll
              for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sr[v]);
              mx = fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(partner_addr, __builtin_bit_cast(int, mx))));
              const float m_up = fmaxf(m[qb], mx);
              const float corr = __builtin_amdgcn_exp2f(m[qb] - m_up);
              l[qb] *= corr;
#pragma unroll
              for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[qb][b][v] *= corr;
              m[qb] = m_up;
              exponentials(sr, -m[qb]);
            }
          }
          if (SUM == SUM_VALU) l[qb] += psum;
        }
        // ---- O^T += V^T . P^T: each V^T fragment feeds all query blocks of the wave
#pragma unroll
        for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            // V^T[32 b + lq][keys 32 kb + 16 s2 + 4 g .. + 3] and the same eight keys on: two transposing reads
            const unsigned char* p = sV + (kb * 32 + s2 * 16) * Sh::V_STRIDE + ((uint32_t)(b * 64) ^ vt_swap) + vt_off;
            const u32x2 lo = read_tr(p), hi = read_tr(p + 8 * Sh::V_STRIDE);
            const u32x4 packed = {lo[0], lo[1], hi[0], hi[1]};
            const bf16x8 vf = __builtin_bit_cast(bf16x8, packed);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
              o[qb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][s2], o[qb][b], 0, 0, 0);
          }
      }

      if (t + 1 < n_tiles) {
        unsigned char* nK = lds + ((t + 1) & 1) * Sh::STAGE;
        store_tile(nK, nK + Sh::K_BYTES);
      }
      __syncthreads();
    };
    // Every load issued so far (the Q fragments among them) has landed before the loop starts: the
    // compiler's wait-count pass otherwise carries "Q may still be in flight" around the loop and makes
    // each tile's first MFMAs wait for the global loads of the NEXT tile issued just before them.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    const int n_full = w.seg_len / AKV;  // tiles with all 64 keys valid
    for (int t = 0; t < n_full; ++t) process_tile(t, std::false_type{});
    if (n_full < n_tiles) process_tile(n_full, std::true_type{});

    // the row sum of every query, in both lanes that share it
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if constexpr (SUM == SUM_VALU) l[qb] += __shfl_xor(l[qb], 32, 64);
      else l[qb] = o[qb][Sh::DB - 1][((DHP % 32) / 8) * 4];
    }
  };

  attend(std::true_type{});
  {
    bool ok = true;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) ok = ok && l[qb] >= 0x1p-100f && l[qb] <= 0x1p100f;  // false for NaN
    // (the barrier also separates the last tile's LDS reads from the general pass's first stores)
    if (__syncthreads_or(wave_active && !ok)) attend(std::false_type{});
  }

  // ---- normalise and store: lane owns a query; registers 4j..4j+3 of block b are
  //      d = 32b + 8j + 4g .. +3, four consecutive columns -> one 8-byte piece.
  // The wave passes its 32 rows through LDS (free after the last tile's barrier; rows 8 bytes longer than the head,
  // so the 8-byte writes of 16 rows and the read-back fall on different banks) and stores them 16 bytes per lane,
  // DHP / 8 lanes per row: a store instruction then touches 4 to 8 rows where direct 8-byte stores touch 32, a
  // quarter of the cache requests for the same bytes.
  if constexpr (QB == 1) {
    if (wave_active) {
      constexpr int ROWB = DHP * 2 + 8, NCH = DHP / 8;
      unsigned char* so = lds + wave * 32 * ROWB;
      const float inv = 1.0f / l[0];  // (rows past the segment end: never stored)
#pragma unroll
      for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (b * 32 + 8 * j >= DHP) continue;  // the spare rows of the last O^T block
          const u32x2 pk = {pack_bf16x2(o[0][b][4 * j] * inv, o[0][b][4 * j + 1] * inv),
                            pack_bf16x2(o[0][b][4 * j + 2] * inv, o[0][b][4 * j + 3] * inv)};
          *(u32x2*)(so + lq * ROWB + (b * 32 + 8 * j + 4 * g) * 2) = pk;
        }
      __builtin_amdgcn_wave_barrier();
      bf16_t* obase = (bf16_t*)a.out + (size_t)(w.q0 + wave * 32) * a.ld_o + head * DHP;
#pragma unroll
      for (int p = 0; p < (32 * NCH + 63) / 64; ++p) {
        const int item = min(p * 64 + lane, 32 * NCH - 1), row = item / NCH, ch = item % NCH;
        const u32x2 lo = *(const u32x2*)(so + row * ROWB + ch * 16), hi = *(const u32x2*)(so + row * ROWB + ch * 16 + 8);
        if (p * 64 + lane < 32 * NCH && w.q0 + wave * 32 + row < seg_end)
          *(u32x4*)(obase + (size_t)row * a.ld_o + ch * 8) = u32x4{lo[0], lo[1], hi[0], hi[1]};
      }
    }
    return;
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qrow = w.q0 + (wave * QB + qb) * 32 + lq;
    if (qrow < seg_end) {
      const float inv = 1.0f / l[qb];
      bf16_t* orow = (bf16_t*)a.out + (size_t)qrow * a.ld_o + head * DHP;
#pragma unroll
      for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int d = b * 32 + 8 * j + 4 * g;
          if (d < DHP) {
            const u32x2 pk = {pack_bf16x2(o[qb][b][4 * j] * inv, o[qb][b][4 * j + 1] * inv),
                              pack_bf16x2(o[qb][b][4 * j + 2] * inv, o[qb][b][4 * j + 3] * inv)};
            *(u32x2*)(orow + d) = pk;
          }
        }
    }
  }
}

}  // namespace

int attention_q_block(int dtype_bf16, int dh_pad) { return !dtype_bf16 ? 64 : 128; }  // 32 * QB * NW

hipError_t launch_attention_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_work <= 0) return hipSuccess;
  if ((a.qkv_rows == 0 && a.ld_qkv % 8 != 0) || a.ld_o % 8 != 0) return hipErrorInvalidValue;
  const dim3 grid(((a.n_work + 7) / 8) * 8, a.heads);
#define VIT_ATTN(DHP, QB, NW)                                                                            \
  do {                                                                                                 \
    constexpr int smem = 2 * AttnShape<DHP, QB, NW>::STAGE;                                            \
    auto kfn = attention_bf16_kernel<DHP, QB, NW>;                                                     \
    static LdsLimitOnce lds_limit; /* raised once per kernel and device */                             \
    if (hipError_t e = lds_limit.ensure((const void*)kfn, smem); e != hipSuccess) return e;            \
    hipLaunchKernelGGL(kfn, grid, dim3(AttnShape<DHP, QB, NW>::ANT), smem, s, a);                      \
  } while (0)
  switch (a.dh_pad) {
    case 64: VIT_ATTN(64, 1, 4); break;
    case 72: VIT_ATTN(72, 1, 4); break;
    case 80: VIT_ATTN(80, 1, 4); break;
    case 96: VIT_ATTN(96, 1, 4); break;
    case 128: VIT_ATTN(128, 1, 4); break;
    default: return hipErrorInvalidValue;
  }
#undef VIT_ATTN
  return hipGetLastError();
}

}  // namespace vitenc
