// Dense blocks of the neighbour aggregation on the matrix cores (Algorithm 1, the AGGREGATE line, for
// the part of a power-law graph that is dense once rows and columns are ordered by degree).
//
// One workgroup per (item, 128-column half of the rows' width).  An item owns the 128 x 128 fp32
// accumulator tile of one row block (in registers) and walks over its dense blocks (at most 32): for every
// block it loads the 64 source rows of the block's column slots (current or historical buffer by the source's
// chunk, Section 3.3; zero for padding slots and for unselected sources of a backward launch, Section 3.4)
// and multiplies, acc += W_hi . H + W_lo . H, the weights being kept as the nearest bf16 and the bf16 of the
// remainder (16 mantissa bits, as in the sparse kernel).  Blocks whose columns all come from an unselected
// chunk are skipped in a backward launch, items with no selected block leave without writing (the reduce
// kernel applies the same test).
//
// One kernel, two sources of the weights.  When the library computes them itself, w(v, u) = s_row(v) s_col(u),
// a block is a 128 x 64 bit pattern plus scales (the benchmark configurations).  Weights given by the caller
// are kept as two 128 x 64 bf16 tiles per block, written once by an expand kernel in the order the matrix
// instruction wants them: [32-row group][16-column step][lane][8 values], so that a wave's A fragment is one
// coalesced 16-byte load per lane.
#include "common.h"

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int DH = 128;      // columns one workgroup owns
constexpr int TILE_ELEMS = kDenseRB * kDenseCB;  // one weight tile in memory
constexpr int HQ_BUF = (kDenseCB / 8) * DH;      // 16-byte words of one source-row buffer in LDS

__device__ inline bool masks_meet(const ChunkMask &x, const ChunkMask &y) {
  return ((x.w[0] & y.w[0]) | (x.w[1] & y.w[1]) | (x.w[2] & y.w[2]) | (x.w[3] & y.w[3])) != 0;
}

// tiles[b] (cleared beforehand) <- entries of block b; one workgroup per block.  Cell (r, c) of a tile sits at
// fragment order: row group r / 32, column step c / 16, lane 32 ((c / 8) % 2) + r % 32, value c % 8.
__global__ __launch_bounds__(256) void dense_expand_kernel(const int64_t *blk_e0, const uint16_t *ent_pos,
                                                          const uint32_t *ent_w, uint16_t *tiles) {
  const int64_t b = blockIdx.x;
  uint16_t *hi = tiles + (size_t)b * 2 * TILE_ELEMS, *lo = hi + TILE_ELEMS;
  for (int64_t e = blk_e0[b] + threadIdx.x; e < blk_e0[b + 1]; e += 256) {
    const uint32_t pos = ent_pos[e], w = ent_w[e];
    if (pos == 0xffffu) continue;  // padding of the entry list
    const int r = (int)(pos >> 8), c = (int)(pos & 255u);
    const int at = ((((r >> 5) * (kDenseCB / 16) + (c >> 4)) * 64 + ((c >> 3) & 1) * 32 + (r & 31)) << 3) + (c & 7);
    hi[at] = (uint16_t)(w & 0xffffu);
    lo[at] = (uint16_t)(w >> 16);
  }
}

// TILES == false: weights of the form w(v, u) = s(v) * s(u) (the normalisation of Section 2.1 computed by the
// library itself).  A block is then a 0/1 pattern, kept as 128 x 64 bits, and
//     out[v] = s(v) * sum_u P(v, u) * s(u) * h(u).
// TILES == true: the A fragments are loaded ready-made from the block's two weight tiles.
// What this kernel has to save is vector instructions: a matrix instruction keeps a SIMD's vector port busy
// for about half of its 32 cycles, so a loop with more than four vector instructions per matrix instruction
// is bound by instruction issue, not by the matrix cores.
//  * A wave owns 32 rows x 128 columns of the accumulator tile, so the A operand of its products is private
//    to it and never goes through LDS.  Pattern blocks: a lane keeps the 64 pattern bits of its row in two
//    registers and makes each A fragment of v_mfma_f32_32x32x16_bf16 (its row, eight consecutive columns) by
//    masking the packed column scales (nearest bf16 and the bf16 of the remainder, one broadcast 16-byte LDS
//    word each) with the masks of the pattern byte, which come from a 256-entry table in LDS.  Tile blocks:
//    the eight fragments of a block (four k-steps, upper and lower part) are eight 16-byte loads per lane.
//  * The 64 source rows of a block are loaded row-wise: a wave takes 16 of them, a lane two columns of each
//    (one 256-byte request per row; the row's address is a broadcast LDS read of a table resolved once per
//    item: current or historical buffer by the source's chunk, a row of zeros for padding slots and - in a
//    backward launch - unselected sources).  A lane then holds its columns of eight consecutive source pairs,
//    i.e. two complete B fragments per column, and stores them as 16-byte words [quad of pairs][column slot]; a
//    B fragment is one 16-byte read.  Column slot s holds column 2s (s < 64) or 2(s - 64) + 1, so that the lanes
//    of a store and of a read touch consecutive words (no bank conflicts); the accumulator tiles inherit that
//    order and tiles ni, ni + 2 leave as pairs of neighbouring columns.
//  * The source rows alternate between two LDS buffers, which leaves one barrier per block.
template <bool TILES>
__global__ __launch_bounds__(256, 2) void spmm_dense_blocks_kernel(const DenseArgs a) {
  constexpr int NI = DH / 32;
  constexpr int S = TILES ? 2 : 3;  // blocks whose loads are in flight (register slots; a tile block carries 32 more registers)
  constexpr int KS = kDenseCB / 16; // k-steps of a block
  constexpr int CP = kDenseCB / 2;  // column pairs of a block
  constexpr int WR = kDenseCB / 4;  // source rows one wave loads
  static_assert(DH == 128 && kDenseCB == 64 && kDenseRB == 128, "lane mapping below");
  extern __shared__ __attribute__((aligned(16))) unsigned char dense_smem[];
  u32x4 *Hq = reinterpret_cast<u32x4 *>(dense_smem);                    // [2 buffers][8 quads][DH]: pairs 4q .. 4q+3 of one column
  uint64_t *rows = reinterpret_cast<uint64_t *>(Hq + 2 * HQ_BUF);       // [blocks][64] address of every source row (at column col0)
  uint32_t *cs_hi = reinterpret_cast<uint32_t *>(rows + kDenseMaxItemBlocks * kDenseCB);  // [blocks][32 column pairs]: nearest bf16 of the two scales
  uint32_t *cs_lo = cs_hi + kDenseMaxItemBlocks * CP;                   // the same for the remainders
  uint32_t *lut = cs_lo + kDenseMaxItemBlocks * CP;                     // [256][4]: pattern byte -> 16-bit masks of its eight cells
  int32_t *m_cb = reinterpret_cast<int32_t *>(TILES ? cs_hi : lut + 256 * 4);  // the three tables above are the pattern blocks' only
  int32_t *act = m_cb + kDenseMaxItemBlocks;                            // the item's selected blocks, in order

  int item = blockIdx.x, half = blockIdx.y;
  // Both halves of an item read the same weights (32 KB of tiles per block; little for pattern blocks, which
  // lose nothing by it).  Workgroups go to the eight XCDs in turn, so in a one-dimensional grid the pairs
  // (item, half 0) and (item, half 1) are put eight apart: same XCD, started together, and the second one finds
  // the weights in that XCD's L2.
  if (a.d > DH) {
    item = (int)(blockIdx.x >> 4) * 8 + (int)(blockIdx.x & 7u);
    half = (int)(blockIdx.x >> 3) & 1;
    if (item >= a.n_items) return;  // whole workgroup: the grid is rounded up to groups of eight items
  }
  const int col0 = half * DH;
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
  if constexpr (!TILES) {
#pragma unroll
    for (int t = 0; t < 4; ++t)  // cells 2t (lower half-word) and 2t + 1 of pattern byte tid
      lut[tid * 4 + t] = ((((uint32_t)tid >> (2 * t)) & 1u) ? 0xffffu : 0u) | ((((uint32_t)tid >> (2 * t + 1)) & 1u) ? 0xffff0000u : 0u);
  }
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
    if constexpr (!TILES) {
#pragma unroll
      for (int q = 0; q < NP; ++q) {  // column pair (2i, 2i + 1) of a block; the scale of a padding slot is zero
        const int i = tid + 256 * q;
        const int64_t slot = i < nb * CP ? (int64_t)m_cb[i >> 5] * kDenseCB + 2 * (i & 31) : 0;
        sc[q][0] = a.colscale[slot];
        sc[q][1] = a.colscale[slot + 1];
      }
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
    for (int q = 0; q < (TILES ? 0 : NP); ++q) {
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
  struct AOperand {
    u32x2 bits;               // pattern blocks: this lane's row, columns 0..31, 32..63
    u32x4 hi[TILES ? KS : 1]; // tile blocks: this lane's A fragment of every k-step, nearest bf16 ...
    u32x4 lo[TILES ? KS : 1]; // ... and the remainder's
  } A[S];
  auto issue = [&](int bi, int u) {
    if constexpr (TILES) {
      const u32x4 *tile = reinterpret_cast<const u32x4 *>(a.tiles + (size_t)(b0 + bi) * 2 * TILE_ELEMS) + (wave * KS) * 64 + lane;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        A[u].hi[ks] = tile[ks * 64];
        A[u].lo[ks] = tile[TILE_ELEMS / 8 + ks * 64];
      }
    } else {
      A[u].bits = *reinterpret_cast<const u32x2 *>(a.bits + (size_t)(b0 + bi) * 256 + 2 * (wm + r32));
    }
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
  // acc += W_hi H + W_lo H (pattern blocks: W_hi = pattern . upper scales, W_lo = pattern . lower scales); the
  // operands of the next k-step are read from LDS while the current one is multiplied
  auto multiply = [&](int bi, const AOperand &w, const u32x4 *H) {
    const uint32_t wsh[2] = {w.bits[0] >> (8 * g), w.bits[1] >> (8 * g)};  // this lane's eight columns of a k-step start at bit 0 / 16
    const u32x4 *ch = reinterpret_cast<const u32x4 *>(cs_hi + bi * CP + g * 4);
    const u32x4 *cl = reinterpret_cast<const u32x4 *>(cs_lo + bi * CP + g * 4);
    u32x4 fb[2][NI], sh[2], sl[2], m4[2];
    auto frags = [&](int ks, int f) {
      if constexpr (!TILES) {
        const uint32_t byte = __builtin_amdgcn_ubfe(wsh[ks >> 1], (ks & 1) * 16, 8);  // this lane's eight cells
        m4[f] = *reinterpret_cast<const u32x4 *>(lut + byte * 4);
        sh[f] = ch[2 * ks];
        sl[f] = cl[2 * ks];
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) fb[f][ni] = H[(2 * ks + g) * DH + ni * 32 + r32];
    };
    frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int f = ks & 1;
      if (ks + 1 < KS) frags(ks + 1, f ^ 1);
      bf16x8 fh, fl;
      if constexpr (TILES) {
        fh = __builtin_bit_cast(bf16x8, w.hi[ks]);
        fl = __builtin_bit_cast(bf16x8, w.lo[ks]);
      } else {
        fh = __builtin_bit_cast(bf16x8, sh[f] & m4[f]);
        fl = __builtin_bit_cast(bf16x8, sl[f] & m4[f]);
      }
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
        const AOperand w = A[u];
        stage(u, buffer(i + u));
        __syncthreads();  // the source rows are in place
        if constexpr (TILES) {  // the fragments stay in their slot until they are used up: no second copy in registers
          multiply(act[i + u], A[u], buffer(i + u));
          issue(act[i + S + u], u);
        } else {
          issue(act[i + S + u], u);
          multiply(act[i + u], w, buffer(i + u));
        }
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
        const AOperand w = A[u];
        stage(u, buffer(i + u));
        __syncthreads();
        if constexpr (TILES) {
          multiply(act[i + u], A[u], buffer(i + u));
          if (i + S + u < na) issue(act[i + S + u], u);
        } else {
          if (i + S + u < na) issue(act[i + S + u], u);
          multiply(act[i + u], w, buffer(i + u));
        }
      }
    }
  }
  float *P = a.partial + (size_t)item * kDenseRB * a.d + col0;
  float rsv[16];  // all loads before the first store: the stores may alias them for all the compiler knows
  if constexpr (TILES) {  // the tiles hold the complete weights
#pragma unroll
    for (int t = 0; t < 16; ++t) rsv[t] = 1.f;
  } else {
    const float *rs = a.rowscale + (size_t)a.item_rb[item] * kDenseRB;  // zero past the last row of the chunk
#pragma unroll
    for (int t = 0; t < 16; ++t) rsv[t] = rs[wm + 8 * (t >> 2) + 4 * g + (t & 3)];
  }
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
  if (!a.zero_row || !a.colslot || !a.src_sel || !a.partial || (a.bits ? !a.colscale || !a.rowscale : !a.tiles))
    return hipErrorInvalidValue;  // the kernel reads all of these without a test of its own
  // source-row buffers, row addresses, block tables; the pattern blocks add their column scales and the mask table
  const size_t common = (size_t)2 * HQ_BUF * 16 + (size_t)kDenseMaxItemBlocks * kDenseCB * sizeof(uint64_t) +
                        (2 * kDenseMaxItemBlocks + 1) * sizeof(int32_t);
  const size_t smem = common + (a.bits ? (size_t)kDenseMaxItemBlocks * kDenseCB * sizeof(uint32_t) + 256 * 4 * sizeof(uint32_t) : 0);
  const auto kernel = a.bits ? spmm_dense_blocks_kernel<false> : spmm_dense_blocks_kernel<true>;
  static bool attr_done[2] = {false, false};
  if (!attr_done[a.bits ? 0 : 1]) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_done[a.bits ? 0 : 1] = true;
  }
  const bool paired = a.d > DH;  // see the kernel: one-dimensional grid, the halves of an item on one XCD
  const dim3 grid = paired ? dim3((unsigned)((a.n_items + 7) / 8 * 16)) : dim3((unsigned)a.n_items, (unsigned)(a.d / DH));
  hipLaunchKernelGGL(kernel, grid, dim3(256), smem, s, a);
  return (int)hipGetLastError();
}

// Diagnostic for CPU tests of the check above: 1 when the launcher refuses a launch whose operand `missing` is absent
// (0 zero row, 1 column slots, 2 selected source table, 3 partial tiles, 4 column scales (pattern blocks) or weight
// tiles, 5 row scales (pattern blocks only)), 0 when it would launch, -1 for an unknown operand.  Nothing is launched:
// the other operands are placeholder addresses that a refused launch never reads.
extern "C" int gnnstage_debug_dense_rejects(int32_t missing, int32_t pattern_blocks) {
  if (missing < 0 || missing > 5 || (missing == 5 && !pattern_blocks)) return -1;
  static char placeholder[16];
  DenseArgs a{};
  a.n_items = 1;
  a.d = 128;
  a.zero_row = placeholder;
  a.colslot = reinterpret_cast<const uint32_t *>(placeholder);
  a.src_sel = placeholder;
  a.partial = reinterpret_cast<float *>(placeholder);
  if (pattern_blocks) {
    a.bits = reinterpret_cast<const uint32_t *>(placeholder);
    a.colscale = reinterpret_cast<const float *>(placeholder);
    a.rowscale = reinterpret_cast<const float *>(placeholder);
  } else {
    a.tiles = reinterpret_cast<const bf16_t *>(placeholder);
  }
  switch (missing) {
    case 0: a.zero_row = nullptr; break;
    case 1: a.colslot = nullptr; break;
    case 2: a.src_sel = nullptr; break;
    case 3: a.partial = nullptr; break;
    case 4: if (pattern_blocks) a.colscale = nullptr; else a.tiles = nullptr; break;
    default: a.rowscale = nullptr; break;
  }
  return launch_spmm_dense(a, nullptr) == (int)hipErrorInvalidValue ? 1 : 0;
}

int launch_dense_expand(const int64_t *blk_e0, const uint16_t *ent_pos, const uint32_t *ent_w, void *tiles, int64_t n_blocks,
                        hipStream_t s) {
  if (n_blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(dense_expand_kernel, dim3((unsigned)n_blocks), dim3(256), 0, s, blk_e0, ent_pos, ent_w,
                     static_cast<uint16_t *>(tiles));
  return (int)hipGetLastError();
}
