// Dense blocks of the neighbour aggregation on the matrix cores (Algorithm 1, the AGGREGATE line, for
// the part of a power-law graph that is dense once rows and columns are ordered by degree).
//
// Two kernels.  When the library computes the weights itself, w(v, u) = s_row(v) s_col(u), a block is a
// 128 x 64 bit pattern plus scales (spmm_dense_r1_kernel, described there; the benchmark configurations).
// Weights given by the caller (spmm_dense_kernel, described here): every dense block is kept in memory as two
// 128 x 64 bf16 tiles, the nearest bf16 of every weight and the bf16 of the remainder (weights keep 16 mantissa
// bits, as in the sparse kernel); an expand kernel writes them once from the block's entry list when the stage
// is created.
//
// One workgroup per (item, 128-column half of the rows' width).  An item owns the 128 x 128 fp32
// accumulator tile of one row block (in registers) and walks over its dense blocks.  For every block it
//   * copies the two weight tiles to LDS (16-byte pieces, rows padded to 144 bytes),
//   * loads the 64 source rows of the block's column slots (current or historical buffer by the
//     source's chunk, Section 3.3; zero for padding slots and for unselected sources of a backward
//     launch, Section 3.4) and stores them to LDS with consecutive source pairs interleaved, which makes
//     the k-contiguous B fragments of v_mfma_f32_32x32x16_bf16 four 4-byte reads,
//   * multiplies: acc += W_hi . H + W_lo . H.
// The loads of the next block are issued before the current one is multiplied.  Blocks whose columns
// all come from an unselected chunk are skipped in a backward launch, items with no selected block leave
// without writing (the reduce kernel applies the same test).
#include "common.h"

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int A_PITCH = 72;  // bf16 elements per weight-tile row in LDS: 144 bytes keep 16-byte fragment reads conflict-free
constexpr int DH = 128;      // columns one workgroup owns
constexpr int TILE_ELEMS = kDenseRB * kDenseCB;  // one weight tile in memory (row-major, no padding)
constexpr int HQ_BUF = (kDenseCB / 8) * DH;      // 16-byte words of one source-row buffer of the pattern kernel

__device__ inline bool masks_meet(const ChunkMask &x, const ChunkMask &y) {
  return ((x.w[0] & y.w[0]) | (x.w[1] & y.w[1]) | (x.w[2] & y.w[2]) | (x.w[3] & y.w[3])) != 0;
}

// tiles[b] (cleared beforehand) <- entries of block b; one workgroup per block
__global__ __launch_bounds__(256) void dense_expand_kernel(const int64_t *blk_e0, const uint16_t *ent_pos,
                                                          const uint32_t *ent_w, uint16_t *tiles) {
  const int64_t b = blockIdx.x;
  uint16_t *hi = tiles + (size_t)b * 2 * TILE_ELEMS, *lo = hi + TILE_ELEMS;
  for (int64_t e = blk_e0[b] + threadIdx.x; e < blk_e0[b + 1]; e += 256) {
    const uint32_t pos = ent_pos[e], w = ent_w[e];
    if (pos == 0xffffu) continue;  // padding of the entry list
    const int at = (int)(pos >> 8) * kDenseCB + (int)(pos & 255u);
    hi[at] = (uint16_t)(w & 0xffffu);
    lo[at] = (uint16_t)(w >> 16);
  }
}

__global__ __launch_bounds__(256, 2) void spmm_dense_kernel(const DenseArgs a) {
  constexpr int NI = 2;              // 32-column tiles per wave (a wave owns 64 x 64 of the 128 x 128 tile)
  constexpr int GROUPS = DH / 8;     // 16-byte pieces per source half-row
  constexpr int SETS = 64 / GROUPS;  // source pairs one wave instruction covers
  constexpr int PPL = 8 / SETS;      // source pairs per lane (a wave stages 8 of the 32 pairs)
  extern __shared__ __attribute__((aligned(16))) unsigned char dense_smem[];
  bf16_t *A_hi = reinterpret_cast<bf16_t *>(dense_smem);
  bf16_t *A_lo = A_hi + kDenseRB * A_PITCH;
  uint32_t *Hp = reinterpret_cast<uint32_t *>(A_lo + kDenseRB * A_PITCH);  // [32 source pairs][DH] interleaved pairs
  uint32_t *ids = Hp + 32 * DH;                                           // [blocks of the item][64] column slots
  int32_t *m_cb = reinterpret_cast<int32_t *>(ids + kDenseMaxItemBlocks * kDenseCB);

  const int item = blockIdx.x;
  const int col0 = blockIdx.y * DH;
  const bool drop = a.src_unsel == nullptr;
  if (drop && !masks_meet(a.item_chunks[item], a.mask)) return;  // whole workgroup
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const uint32_t vmask = (1u << a.vbits) - 1u;
  const int64_t b0 = a.item_b0[item];
  const int nb = a.item_nb[item];
  const bf16_t *src_sel = static_cast<const bf16_t *>(a.src_sel) + col0;
  const bf16_t *src_unsel = drop ? nullptr : static_cast<const bf16_t *>(a.src_unsel) + col0;
  const size_t ld = (size_t)a.src_ld;

  // the item's column slots go to LDS once, so that all loads of a block can be issued at once
  if (tid < nb) m_cb[tid] = a.blk_cb[b0 + tid];
  __syncthreads();
  for (int i = tid; i < nb * kDenseCB; i += 256) ids[i] = a.colslot[(int64_t)m_cb[i >> 6] * kDenseCB + (i & 63)];
  __syncthreads();

  f32x16 acc[2][NI];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[mi][ni][t] = 0.f;

  const int ng = lane % GROUPS, set = lane / GROUPS;
  // registers that carry one block from its loads to LDS: the source rows of this wave's 8 pairs and this
  // thread's 16-byte pieces of the two weight tiles
  u32x4 x0[PPL], x1[PPL], th[4], tl[4];
  auto next_active = [&](int bi) {  // wave-uniform: slot 0 of a block is never padding
    while (bi < nb && drop && !mask_test(a.mask, ids[bi * kDenseCB] >> a.vbits)) ++bi;
    return bi;
  };
  auto issue = [&](int bi) {
    const u32x4 *tile = reinterpret_cast<const u32x4 *>(a.tiles + (size_t)(b0 + bi) * 2 * TILE_ELEMS);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      th[j] = tile[tid + 256 * j];
      tl[j] = tile[TILE_ELEMS / 8 + tid + 256 * j];
    }
#pragma unroll
    for (int j = 0; j < PPL; ++j) {
      const int kp = wave * 8 + j * SETS + set;
      const uint32_t pc0 = ids[bi * kDenseCB + 2 * kp], pc1 = ids[bi * kDenseCB + 2 * kp + 1];
      x0[j] = u32x4{0u, 0u, 0u, 0u};
      x1[j] = u32x4{0u, 0u, 0u, 0u};
      if (pc0 != 0xffffffffu) {
        const bool sel = mask_test(a.mask, pc0 >> a.vbits);
        if (sel || !drop) x0[j] = *reinterpret_cast<const u32x4 *>((sel ? src_sel : src_unsel) + (size_t)(pc0 & vmask) * ld + ng * 8);
      }
      if (pc1 != 0xffffffffu) {
        const bool sel = mask_test(a.mask, pc1 >> a.vbits);
        if (sel || !drop) x1[j] = *reinterpret_cast<const u32x4 *>((sel ? src_sel : src_unsel) + (size_t)(pc1 & vmask) * ld + ng * 8);
      }
    }
  };

  int cur = next_active(0);
  if (cur < nb) issue(cur);
  while (cur < nb) {
    const int nxt = next_active(cur + 1);
    __syncthreads();  // the previous block's fragment reads are done
    // weight tiles: piece i covers row i / 8, columns 8 * (i % 8) ..
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = tid + 256 * j;
      const int at = (i >> 3) * A_PITCH + (i & 7) * 8;
      *reinterpret_cast<u32x4 *>(A_hi + at) = th[j];
      *reinterpret_cast<u32x4 *>(A_lo + at) = tl[j];
    }
    // source rows: word n of pair kp holds (row 2kp, row 2kp+1) at column n
#pragma unroll
    for (int j = 0; j < PPL; ++j) {
      const int kp = wave * 8 + j * SETS + set;
      u32x4 lo4, hi4;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        lo4[2 * q] = __builtin_amdgcn_perm(x1[j][q], x0[j][q], 0x05040100u);      // column 2q of this lane's eight
        lo4[2 * q + 1] = __builtin_amdgcn_perm(x1[j][q], x0[j][q], 0x07060302u);  // column 2q + 1
        hi4[2 * q] = __builtin_amdgcn_perm(x1[j][q + 2], x0[j][q + 2], 0x05040100u);
        hi4[2 * q + 1] = __builtin_amdgcn_perm(x1[j][q + 2], x0[j][q + 2], 0x07060302u);
      }
      u32x4 *dst = reinterpret_cast<u32x4 *>(Hp + (size_t)kp * DH + ng * 8);
      dst[0] = lo4;
      dst[1] = hi4;
    }
    __syncthreads();  // weights and source rows are in place
    if (nxt < nb) issue(nxt);  // the next block's loads fly while this one is multiplied
#pragma unroll
    for (int ks = 0; ks < kDenseCB / 16; ++ks) {
      bf16x8 fh[2], fl[2], fb[NI];
      const int koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) {
        fh[mi] = *reinterpret_cast<const bf16x8 *>(&A_hi[(wm + mi * 32 + (lane & 31)) * A_PITCH + koff]);
        fl[mi] = *reinterpret_cast<const bf16x8 *>(&A_lo[(wm + mi * 32 + (lane & 31)) * A_PITCH + koff]);
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        u32x4 w4;
#pragma unroll
        for (int j = 0; j < 4; ++j) w4[j] = Hp[(size_t)(ks * 8 + (lane >> 5) * 4 + j) * DH + wn + ni * 32 + (lane & 31)];
        fb[ni] = __builtin_bit_cast(bf16x8, w4);
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fh[mi], fb[ni], acc[mi][ni], 0, 0, 0);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fl[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    }
    cur = nxt;
  }
  // 32x32 accumulator layout: element t of lane l is row 8*(t/4) + 4*(l/32) + t%4, column l%32
  float *P = a.partial + (size_t)item * kDenseRB * a.d + col0;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const int r = wm + mi * 32 + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
        P[(size_t)r * a.d + wn + ni * 32 + (lane & 31)] = acc[mi][ni][t];
      }
}

// The same product for weights of the form w(v, u) = s(v) * s(u) (the normalisation of Section 2.1 computed
// by the library itself).  A block is then a 0/1 pattern, kept as 128 x 64 bits, and
//     out[v] = s(v) * sum_u P(v, u) * s(u) * h(u).
// What this kernel has to save is vector instructions: a matrix instruction keeps a SIMD's vector port busy
// for about half of its 32 cycles, so a loop with more than four vector instructions per matrix instruction
// is bound by instruction issue, not by the matrix cores.
//  * A wave owns 32 rows x 128 columns of the accumulator tile, so the A operand of its products is private
//    to it and never goes through LDS: a lane keeps the 64 pattern bits of its row in two registers and
//    makes each A fragment of v_mfma_f32_32x32x16_bf16 (its row, eight consecutive columns) by masking the
//    packed column scales (nearest bf16 and the bf16 of the remainder, one broadcast 16-byte LDS word each)
//    with the masks of the pattern byte, which come from a 256-entry table in LDS.
//  * The 64 source rows of a block are loaded row-wise: a wave takes 16 of them, a lane two columns of each
//    (one 256-byte request per row; the row's address is a broadcast LDS read of a table resolved once per
//    item: current or historical buffer by the source's chunk, a row of zeros for padding slots and - in a
//    backward launch - unselected sources).  A lane then holds its columns of eight consecutive source pairs,
//    i.e. two complete B fragments per column, and stores them as 16-byte words [quad of pairs][column slot]; a
//    B fragment is one 16-byte read.  Column slot s holds column 2s (s < 64) or 2(s - 64) + 1, so that the lanes
//    of a store and of a read touch consecutive words (no bank conflicts); the accumulator tiles inherit that
//    order and tiles ni, ni + 2 leave as pairs of neighbouring columns.
//  * The source rows alternate between two LDS buffers, which leaves one barrier per block.
__global__ __launch_bounds__(256, 2) void spmm_dense_r1_kernel(const DenseArgs a) {
  constexpr int NI = DH / 32;
  constexpr int S = 3;              // blocks whose loads are in flight (register slots)
  constexpr int CP = kDenseCB / 2;  // column pairs of a block
  constexpr int WR = kDenseCB / 4;  // source rows one wave loads
  static_assert(DH == 128 && kDenseCB == 64 && kDenseRB == 128, "lane mapping below");
  extern __shared__ __attribute__((aligned(16))) unsigned char dense_smem[];
  u32x4 *Hq = reinterpret_cast<u32x4 *>(dense_smem);                    // [2 buffers][8 quads][DH]: pairs 4q .. 4q+3 of one column
  uint64_t *rows = reinterpret_cast<uint64_t *>(Hq + 2 * HQ_BUF);       // [blocks][64] address of every source row (at column col0)
  uint32_t *cs_hi = reinterpret_cast<uint32_t *>(rows + kDenseMaxItemBlocks * kDenseCB);  // [blocks][32 column pairs]: nearest bf16 of the two scales
  uint32_t *cs_lo = cs_hi + kDenseMaxItemBlocks * CP;                   // the same for the remainders
  uint32_t *lut = cs_lo + kDenseMaxItemBlocks * CP;                     // [256][4]: pattern byte -> 16-bit masks of its eight cells
  int32_t *m_cb = reinterpret_cast<int32_t *>(lut + 256 * 4);
  int32_t *act = m_cb + kDenseMaxItemBlocks;                            // the item's selected blocks, in order

  const int item = blockIdx.x;
  const int col0 = blockIdx.y * DH;
  const bool drop = a.src_unsel == nullptr;
  if (drop && !masks_meet(a.item_chunks[item], a.mask)) return;  // whole workgroup
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave * 32, g = lane >> 5, r32 = lane & 31;
  const uint32_t vmask = (1u << a.vbits) - 1u;
  const int64_t b0 = a.item_b0[item];
  const int nb = a.item_nb[item];
  const bf16_t *src_sel = static_cast<const bf16_t *>(a.src_sel) + col0;
  const bf16_t *src_unsel = drop ? src_sel : static_cast<const bf16_t *>(a.src_unsel) + col0;
  const size_t ld = (size_t)a.src_ld;
  const uint64_t zrow = reinterpret_cast<uint64_t>(a.zero_row);  // 128 zeros are enough for any column half

  if (tid < nb) m_cb[tid] = a.blk_cb[b0 + tid];
#pragma unroll
  for (int t = 0; t < 4; ++t)  // cells 2t (lower half-word) and 2t + 1 of pattern byte tid
    lut[tid * 4 + t] = ((((uint32_t)tid >> (2 * t)) & 1u) ? 0xffffu : 0u) | ((((uint32_t)tid >> (2 * t + 1)) & 1u) ? 0xffff0000u : 0u);
  __syncthreads();
  {  // all loads of the two tables first, in one round trip: up to 8 column slots and 4 column pairs per thread
    constexpr int NQ = kDenseMaxItemBlocks * kDenseCB / 256, NP = kDenseMaxItemBlocks * CP / 256;
    uint32_t pc[NQ];
    float sc[NP][2];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int i = tid + 256 * q;
      pc[q] = i < nb * kDenseCB ? a.colslot[(int64_t)m_cb[i >> 6] * kDenseCB + (i & 63)] : 0xffffffffu;
    }
#pragma unroll
    for (int q = 0; q < NP; ++q) {  // column pair (2i, 2i + 1) of a block; the scale of a padding slot is zero
      const int i = tid + 256 * q;
      const int64_t slot = i < nb * CP ? (int64_t)m_cb[i >> 5] * kDenseCB + 2 * (i & 31) : 0;
      sc[q][0] = a.colscale[slot];
      sc[q][1] = a.colscale[slot + 1];
    }
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int i = tid + 256 * q;
      uint64_t addr = zrow;
      if (pc[q] != 0xffffffffu) {
        const bool sel = mask_test(a.mask, pc[q] >> a.vbits);
        if (sel || !drop) addr = reinterpret_cast<uint64_t>((sel ? src_sel : src_unsel) + (size_t)(pc[q] & vmask) * ld);
      }
      if (i < nb * kDenseCB) rows[i] = addr;
    }
#pragma unroll
    for (int q = 0; q < NP; ++q) {
      const int i = tid + 256 * q;
      uint32_t part[2][2];  // [column of the pair][upper, lower]
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const bf16_t h = (bf16_t)sc[q][c];
        const bf16_t l = (bf16_t)(sc[q][c] - (float)h);
        part[c][0] = __builtin_bit_cast(uint16_t, h);
        part[c][1] = __builtin_bit_cast(uint16_t, l);
      }
      if (i < nb * CP) {
        cs_hi[i] = part[0][0] | (part[1][0] << 16);
        cs_lo[i] = part[0][1] | (part[1][1] << 16);
      }
    }
  }
  __syncthreads();
  if (wave == 0) {  // a block whose first slot resolved to the row of zeros in a backward launch has no selected source
    const bool on = lane < nb && (!drop || rows[(lane < nb ? lane : 0) * kDenseCB] != zrow);
    const uint64_t bal = __ballot(on);
    if (on) act[__popcll(bal & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) act[kDenseMaxItemBlocks] = __popcll(bal);
  }
  __syncthreads();
  const int na = act[kDenseMaxItemBlocks];

  f32x16 acc[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[ni][t] = 0.f;

  // register slots: slot u carries the active block i with i % S == u from its loads to its products.  Every
  // load is unconditional, so the number of younger loads at every wait is a compile-time constant.
  uint32_t x[S][WR];  // columns 2 lane, 2 lane + 1 of the wave's source rows
  u32x2 bits[S];      // the pattern of this lane's row: columns 0..31, 32..63
  auto issue = [&](int bi, int u) {
    bits[u] = *reinterpret_cast<const u32x2 *>(a.bits + (size_t)(b0 + bi) * 256 + 2 * (wm + r32));
    const uint64_t *rp = rows + bi * kDenseCB + wave * WR;  // the same for all lanes: broadcast reads
#pragma unroll
    for (int r = 0; r < WR; ++r)  // device memory, said so: a generic load would also count as an LDS access in the waits
      x[u][r] = *reinterpret_cast<const __attribute__((address_space(1))) uint32_t *>(rp[r] + 4u * (uint32_t)lane);
    __builtin_amdgcn_sched_barrier(0);  // keep the slots' loads in program order (the waits count younger loads)
  };
  // source rows of slot u -> buffer H: the wave's rows are pairs 8 wave .. 8 wave + 7, i.e. quads 2 wave, 2 wave + 1
  auto stage = [&](int u, u32x4 *H) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      u32x4 even, odd;  // columns 2 lane and 2 lane + 1: (row 2p | row 2p + 1 << 16) for the quad's four pairs p
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t p0 = x[u][8 * q + 2 * t], p1 = x[u][8 * q + 2 * t + 1];
        even[t] = __builtin_amdgcn_perm(p1, p0, 0x05040100u);
        odd[t] = __builtin_amdgcn_perm(p1, p0, 0x07060302u);
      }
      u32x4 *dst = H + (2 * wave + q) * DH + lane;  // column slots: the even columns first, then the odd ones
      dst[0] = even;
      dst[DH / 2] = odd;
    }
  };
  // acc += (pattern . upper scales) H + (pattern . lower scales) H; the operands of the next k-step are read
  // from LDS while the current one is multiplied
  auto multiply = [&](int bi, u32x2 w, const u32x4 *H) {
    const uint32_t wsh[2] = {w[0] >> (8 * g), w[1] >> (8 * g)};  // this lane's eight columns of a k-step start at bit 0 / 16
    const u32x4 *ch = reinterpret_cast<const u32x4 *>(cs_hi + bi * CP + g * 4);
    const u32x4 *cl = reinterpret_cast<const u32x4 *>(cs_lo + bi * CP + g * 4);
    u32x4 fb[2][NI], sh[2], sl[2], m4[2];
    auto frags = [&](int ks, int f) {
      const uint32_t byte = __builtin_amdgcn_ubfe(wsh[ks >> 1], (ks & 1) * 16, 8);  // this lane's eight cells
      m4[f] = *reinterpret_cast<const u32x4 *>(lut + byte * 4);
      sh[f] = ch[2 * ks];
      sl[f] = cl[2 * ks];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) fb[f][ni] = H[(2 * ks + g) * DH + ni * 32 + r32];
    };
    frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < kDenseCB / 16; ++ks) {
      const int f = ks & 1;
      if (ks + 1 < kDenseCB / 16) frags(ks + 1, f ^ 1);
      const bf16x8 fh = __builtin_bit_cast(bf16x8, sh[f] & m4[f]), fl = __builtin_bit_cast(bf16x8, sl[f] & m4[f]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fh, __builtin_bit_cast(bf16x8, fb[f][ni]), acc[ni], 0, 0, 0);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fl, __builtin_bit_cast(bf16x8, fb[f][ni]), acc[ni], 0, 0, 0);
    }
  };
  // Block number idx of the item uses buffer idx % 2.  A wave that stores block idx + 2 has passed the barrier of
  // block idx + 1, which every wave reaches only after its products of block idx: one barrier per block is enough.
  auto buffer = [&](int idx) { return Hq + (idx & 1) * HQ_BUF; };

  // prologue, steady groups of S blocks (every refill unconditional), tail
  int i = 0;
  if (na >= 2 * S) {
#pragma unroll
    for (int u = 0; u < S; ++u) issue(act[u], u);
    for (; i + 2 * S <= na; i += S) {
#pragma unroll
      for (int u = 0; u < S; ++u) {
        const u32x2 w = bits[u];
        stage(u, buffer(i + u));
        __syncthreads();  // the source rows are in place
        issue(act[i + S + u], u);
        multiply(act[i + u], w, buffer(i + u));
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < S; ++u)
      if (u < na) issue(act[u], u);
  }
  for (; i < na; i += S) {
#pragma unroll
    for (int u = 0; u < S; ++u) {
      if (i + u < na) {
        const u32x2 w = bits[u];
        stage(u, buffer(i + u));
        __syncthreads();
        if (i + S + u < na) issue(act[i + S + u], u);
        multiply(act[i + u], w, buffer(i + u));
      }
    }
  }
  float *P = a.partial + (size_t)item * kDenseRB * a.d + col0;
  const float *rs = a.rowscale + (size_t)a.item_rb[item] * kDenseRB;  // zero past the last row of the chunk
  float rsv[16];  // all loads before the first store: the stores may alias them for all the compiler knows
#pragma unroll
  for (int t = 0; t < 16; ++t) rsv[t] = rs[wm + 8 * (t >> 2) + 4 * g + (t & 3)];
#pragma unroll
  for (int ni = 0; ni < NI / 2; ++ni)  // tile ni holds the even columns 2 (32 ni + lane), tile ni + 2 the odd ones next to them
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const int r = wm + 8 * (t >> 2) + 4 * g + (t & 3);
      *reinterpret_cast<f32x2 *>(&P[(size_t)r * a.d + 2 * (ni * 32 + r32)]) = f32x2{acc[ni][t] * rsv[t], acc[ni + 2][t] * rsv[t]};
    }
}

}  // namespace

int launch_spmm_dense(const DenseArgs &a, hipStream_t s) {
  if (a.n_items <= 0) return hipSuccess;
  if (a.d != 128 && a.d != 256) return hipErrorInvalidValue;
  const size_t smem = (size_t)2 * kDenseRB * A_PITCH * sizeof(bf16_t) + (size_t)32 * DH * sizeof(uint32_t) +
                      (size_t)kDenseMaxItemBlocks * kDenseCB * sizeof(uint32_t) + kDenseMaxItemBlocks * sizeof(int32_t);
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(spmm_dense_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)smem);
    attr_done = true;
  }
  if (a.bits) {
    const size_t smem1 = (size_t)2 * HQ_BUF * 16 + (size_t)kDenseMaxItemBlocks * kDenseCB * (sizeof(uint64_t) + sizeof(uint32_t)) +
                         (size_t)256 * 4 * sizeof(uint32_t) + (2 * kDenseMaxItemBlocks + 1) * sizeof(int32_t);
    static bool attr1_done = false;
    if (!attr1_done) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(spmm_dense_r1_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem1);
      attr1_done = true;
    }
    hipLaunchKernelGGL(spmm_dense_r1_kernel, dim3((unsigned)a.n_items, (unsigned)(a.d / DH)), dim3(256), smem1, s, a);
    return (int)hipGetLastError();
  }
  hipLaunchKernelGGL(spmm_dense_kernel, dim3((unsigned)a.n_items, (unsigned)(a.d / DH)), dim3(256), smem, s, a);
  return (int)hipGetLastError();
}

int launch_dense_expand(const int64_t *blk_e0, const uint16_t *ent_pos, const uint32_t *ent_w, void *tiles, int64_t n_blocks,
                        hipStream_t s) {
  if (n_blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(dense_expand_kernel, dim3((unsigned)n_blocks), dim3(256), 0, s, blk_e0, ent_pos, ent_w,
                     static_cast<uint16_t *>(tiles));
  return (int)hipGetLastError();
}
