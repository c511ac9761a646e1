// Tile kernel for O = W_s x I (Section 5, "GPU Implementation"), bf16 inputs with fp32
// accumulation: v_mfma_f32_32x32x16_bf16.
//
// The level of the pattern this kernel uses is the outermost one: every nonzero of G_o is a
// TM x TK block of W_s (TM = |G_r.U| |G_i.U| |G_b.U| rows, TK = |G_r.V| |G_i.V| |G_b.V| columns), and the
// rows of I one block multiplies are consecutive (tile skipping through G_o's adjacency, as in
// Section 5).  Inside a block the weights are stored dense, with zeros where the inner graphs
// have no edge: the bf16 matrix core has the room (a 32x32x16 MFMA issues every ~35 cycles), and
// in return the B operand needs no gather, every row of a tile row is useful to every MFMA, and
// a workgroup can stage I in LDS ONCE for all its tile rows -- the register-streaming family is
// bound by the bytes of I that cross the L1 path (every cluster and G_i vertex loads its own).
//
// Workgroup = 4 consecutive tile rows x 64 columns, 8 waves.  Stage = one tile column that any of
// the four tile rows has (host table, ascending): producer waves load its TKP rows x 64 columns of I
// with 16-byte loads (a lane takes 8 rows x 8 columns), transpose them in registers (v_perm_b32)
// into, per column, eight consecutive contraction steps (what one lane feeds the matrix core), and
// write them to LDS as [8-row block][column position][16 bytes], position = column ^ (2 * ((column / 16) % 4) + block % 2):
// the 16-byte writes of 16 neighbouring lanes (8 column octets x 2 blocks, same column offset) then fall
// on 16 different bank groups, while the 32 lanes of a read still cover 512 contiguous bytes.
// Two LDS buffers and one barrier per stage: consumers multiply stage s while producers fill the
// buffer of stage s + 1, with the loads of stage s + 2 in flight (two register sets).
// A consumer wave whose tile row lacks the tile column skips the MFMAs of the stage (its weight
// loads point past the packed buffer and return zeros without a memory access).
// The fused 3x3 convolution runs here too: only the producers' addresses change (stage row k is
// tap k % 9 of channel k / 9 of the zero-padded activations).
// Measured against the register-streaming family on the VGG19 layers in bf16: faster where the
// tiles are dense (density 1/2 on the layers with many columns, by 13-30 %), slower elsewhere;
// never chosen by RBGP_KERNEL_AUTO.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <new>
#include <type_traits>
#include <vector>

#include "rbgp_internal.h"
#include "rbgp_reg_common.h"

using namespace rbgp_reg;

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kInline = 240;

struct TileParams {
  const void *Wp;          // packed weights: [tile row][j_o][TKP / 16][2][TM][8] bf16
  const void *I;           // K x ldI bf16
  void *O;                 // M x ldO fp32, or bf16 bits when obf16 is set
  const int32_t *stages;   // [row groups][max_stages + 4 * d_o]: tile column of every stage, then per consumer wave
                           //   the stage of each tile of its tile row (adjacency-list order = ascending)
  const int32_t *counts;   // [row groups] stages
  int64_t N, ldI, ldO, K;
  int obf16;
  int max_stages;
  int a_o, d_o;
  int TK;
  int tab_bytes;           // LDS bytes of the stage list (a multiple of 16)
  int inl_ok;              // the stage lists and counts of all row groups fit `inl` (then stages / counts are unused):
                           //   saves the copy of the table to LDS and its barrier (measured on the VGG19 conv3 shape:
                           //   21.0 us against 21.3 us)
  int32_t inl[kInline];    // the table above, then [row groups] counts
  int ntiles, RG;          // column tiles of 64, row groups of 4 tile rows
  // Fused 3x3 convolution: I is the zero-padded activation tensor X[channel][image][H + 2][W + 2] (bf16) and row
  // k = 9 * channel + tap of the lowered input is read from it: a tile column is TK / 9 consecutive channels.
  int conv;                // 1: fused convolution
  int conv_w2;             // W + 2 (pixels of a padded image row)
  uint32_t chan_bytes;     // bytes of one channel of X
  int64_t x_bytes;         // bytes of X (< 2^31)
  const int32_t *colbase;  // [ntiles * 8]: byte offset, inside a channel of X, of the first pixel of every group of
                           //   8 columns (8 pixels of one image row: W % 8 == 0); padded to whole tiles
  uint32_t w_bytes;
  uint32_t n_round_bytes;  // N rounded up to 8 columns, in bytes: the extent of the last row of I
};

constexpr int kCW = 64;        // columns per workgroup

template <int NT>
struct RawSet {
  u32x4 r[NT > 0 ? NT : 1][8];
};

// Workgroup = 8 waves: waves 0..3 are consumers (one tile row each: weights from global memory, B
// operands from LDS, MFMAs), waves 4..7 producers (rows of I from global memory to LDS).  The two
// kinds share a SIMD pairwise, so the matrix core runs while the other wave waits for memory, and
// each kind has its own in-order load counter: a consumer's wait for weights never waits for I.
// NC: 16-step blocks of a stage (TKP = 16 * NC), a compile-time constant so that a consumer can hold
// the weights of a whole tile in registers: those of its next tile are requested before the MFMAs
// of the current one.
template <int NC>
__global__ __launch_bounds__(512) void spmm_tile_bf16(TileParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  constexpr int TM = 32;
  constexpr int TKP = 16 * NC;
  constexpr int NBLK = 2 * NC;                 // 8-row blocks of a stage
  constexpr int BUF = NBLK * kCW * 16;         // bytes of one stage in LDS
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  // workgroups are dealt round-robin to the 8 XCDs: the row groups of one column tile share an L2
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int rg = slot % p.RG, nt = (slot / p.RG) * 8 + xcd;
  if (nt >= p.ntiles) return;   // (the whole workgroup)
  const int64_t n0 = int64_t(nt) * kCW;
  // The table of the row group (tile column of every stage, then per consumer wave the stage of each of
  // its tiles) comes from the kernel arguments when it fits them, else it is copied to LDS first
  // (reading it later must not wait for the loads in flight).
  const bool inl = p.inl_ok != 0;
  // (the kernel arguments the epilogue needs, read here: fetched after the loop, they would add scalar-load
  // latencies to the end of every consumer wave)
  void *const out = p.O;
  const int64_t out_ld = p.ldO, out_n = p.N;
  const int out_bf16 = p.obf16;
  const int rec = p.max_stages + 4 * p.d_o;    // words per row group
  const int cnt = inl ? p.inl[p.RG * rec + rg] : p.counts[rg];
  int32_t *const tab = reinterpret_cast<int32_t *>(lds_raw);
  unsigned char *const lds = lds_raw + p.tab_bytes;
  if (!inl) {
    const int32_t *stg = p.stages + int64_t(rg) * rec;
    for (int i = tid; i < rec; i += 512) tab[i] = stg[i];
    __syncthreads();
  }
  const int inl_base = rg * rec;
  auto table = [&](int i) { return inl ? p.inl[inl_base + i] : __builtin_amdgcn_readfirstlane(tab[i]); };

  if (wid >= 4) {
    // ---------------------------------------------------------------- producer
    // Load tasks: (8 rows x 8 columns) pieces of the stage, task t = (block t / 8, column octet t % 8),
    // dealt to the 256 producer threads in rounds; the last round may cover only some of the waves, so
    // the code below exists for both task counts (a wave-uniform choice: every wave's count of loads in
    // flight is a compile-time constant).
    const int ptid = tid - 256;
    constexpr int NTASK = NBLK * 8, FULL = NTASK / 256, REM = NTASK % 256;
    auto producer = [&](auto nt_c) {
      constexpr int NT = decltype(nt_c)::value;
      const int row_bytes = int(p.ldI) * 2;
      // byte offset of every load of this thread inside the stage's descriptor.  Plain product: row of the stage
      // times the row pitch plus the octet's columns.  Fused convolution: stage row k is tap k % 9 of the stage's
      // channel k / 9 -- channel pitch, plus the octet's first pixel in the padded image (host table), plus the
      // shift of the tap (the loads are then 2-byte aligned, which the memory path accepts).
      int l_off[NT > 0 ? NT : 1][8], t_lds[NT > 0 ? NT : 1];
#pragma unroll
      for (int q = 0; q < NT; ++q) {
        const int t = ptid + 256 * q, blk = t >> 3, oct = t & 7;
        const int pix = p.conv ? p.colbase[(nt * 8 + oct)] : 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const int k = blk * 8 + r;
          int off;
          if (p.conv) {
            const int ch = int(uint32_t(k) / 9u), tap = k - 9 * ch;
            const int dy = tap / 3 - 1, dx = tap - 3 * (tap / 3) - 1;
            off = int(uint32_t(ch) * p.chan_bytes) + pix + (dy * p.conv_w2 + dx) * 2;
          } else {
            off = k * row_bytes + oct * 16;   // < 2^30: checked by the host
          }
          l_off[q][r] = t < NTASK ? off : kOob;
        }
        t_lds[q] = (blk * kCW + oct * 8) * 16;
      }
      // position swizzle inside a block (see the file header): all tasks of a thread have the same octet
      // and the same block parity (256 / 8 is even)
      const int swz = (((ptid & 7) >> 1) << 1) | ((ptid >> 3) & 1);
      // Loads of stage s (zeros without a memory access past the last stage): the descriptor starts at
      // the stage's first row and the workgroup's first column; its extent ends with the last row of I.
      auto issue_loads = [&](int s, RawSet<NT> &set) {
        const bool live = s < cnt;
        const int v_o = live ? table(s) : 0;
        const int64_t row0 = int64_t(v_o) * p.TK;
        const int64_t rows_left = p.K - row0;      // >= TK
        uint64_t base = reinterpret_cast<uint64_t>(p.I) + uint64_t(row0 * p.ldI + n0) * 2;
        int64_t ext = rows_left > TKP ? int64_t(TKP) * p.ldI * 2
                                      : (rows_left - 1) * p.ldI * 2 + (int64_t(p.n_round_bytes) - n0 * 2);
        if (p.conv) {   // the descriptor starts at the stage's first channel and ends with X
          const int64_t first = int64_t(v_o) * (p.TK / 9) * p.chan_bytes;
          base = reinterpret_cast<uint64_t>(p.I) + uint64_t(first);
          ext = p.x_bytes - first;
        }
        if (!live) ext = 0;
        const __amdgpu_buffer_rsrc_t rb =
            __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(base), 0, int(ext), kRsrcFlags);
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
          for (int r = 0; r < 8; ++r)
            set.r[q][r] = __builtin_amdgcn_raw_buffer_load_b128(rb, l_off[q][r], 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      };
      // transpose the 8 x 8 blocks (dword d of a row holds columns 2d and 2d + 1) and write them to LDS buffer b
      auto to_lds = [&](int b, const RawSet<NT> &set) {
        constexpr unsigned LO = 0x05040100u, HI = 0x07060302u;
        unsigned char *dst = lds + b * BUF;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
          if (ptid + 256 * q < NTASK) {
            const u32x4 *r = set.r[q];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              const u32x4 lo = {__builtin_amdgcn_perm(r[1][d], r[0][d], LO), __builtin_amdgcn_perm(r[3][d], r[2][d], LO),
                                __builtin_amdgcn_perm(r[5][d], r[4][d], LO), __builtin_amdgcn_perm(r[7][d], r[6][d], LO)};
              const u32x4 hi = {__builtin_amdgcn_perm(r[1][d], r[0][d], HI), __builtin_amdgcn_perm(r[3][d], r[2][d], HI),
                                __builtin_amdgcn_perm(r[5][d], r[4][d], HI), __builtin_amdgcn_perm(r[7][d], r[6][d], HI)};
              *reinterpret_cast<u32x4 *>(dst + t_lds[q] + (((2 * d) ^ swz) << 4)) = lo;
              *reinterpret_cast<u32x4 *>(dst + t_lds[q] + (((2 * d + 1) ^ swz) << 4)) = hi;
            }
          }
        }
      };
      // NS register sets: the loads of stages s + 2 .. s + NS are in flight while stage s + 1 moves to LDS.
      // Measured on the VGG19 conv3 shape (us per launch): NS = 1: 18.6, 2: 17.4, 3: 18.6, 6: 20.0 -- one
      // stage of lead hides the latency; more loads in flight only queue in front of the consumers' weight
      // loads (and 64 or more per wave exceed the hardware's load counter: NS = 4 with two tasks, 41.6).
      constexpr int NS = 2;
      RawSet<NT> sets[NS];
      static_for<0, NS>([&](auto ic) { issue_loads(decltype(ic)::value, sets[decltype(ic)::value]); });
      to_lds(0, sets[0]);
      __syncthreads();
      // iteration s: request stage s + NS into the set stage s came from, move stage s + 1 to LDS
      auto pstep = [&](int s, RawSet<NT> &free_set, RawSet<NT> &cur) {
        issue_loads(s + NS, free_set);
        if (s + 1 < cnt) to_lds((s + 1) & 1, cur);
        __syncthreads();
      };
      for (int s = 0; s < cnt; s += NS)
        static_for<0, NS>([&](auto ic) {
          constexpr int i = decltype(ic)::value;
          if (s + i < cnt) pstep(s + i, sets[i], sets[(i + 1) % NS]);
        });
      __builtin_amdgcn_s_waitcnt(0);
    };
    if ((wid - 4) * 64 < REM)
      producer(std::integral_constant<int, FULL + 1>{});
    else
      producer(std::integral_constant<int, FULL>{});
    return;
  }

  // ------------------------------------------------------------------ consumer
  // A consumer walks the tiles of its own tile row only (tile j sits in stage table(max_stages + wave * d_o + j)
  // of the row group) and passes the barriers of the stages in between.
  const int u_o = rg * 4 + wid;
  const int ntile = u_o < p.a_o ? p.d_o : 0;
  const __amdgpu_buffer_rsrc_t rw =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.Wp), 0, p.w_bytes, kRsrcFlags);
  constexpr int FRAG = TKP * TM * 2;       // bytes of one tile's weights
  const int n32 = lane & 31, h2 = lane >> 5;
  const int alane = (h2 * TM + n32) * 16;
  // byte offset inside a block of the lane's column 32 h + n32: position (column ^ key), key from the
  // column's octet and the block parity
  const int boff0 = (n32 ^ ((((n32 >> 3) >> 1) << 1) | h2)) << 4;
  const int boff1 = ((32 + n32) ^ (((((32 + n32) >> 3) >> 1) & 3) << 1 | h2)) << 4;

  f32x16 acc[2];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[h][r] = 0.f;

  // the weights of the tile row's tile j (zeros without a memory access past its last tile)
  auto issue_weights = [&](int j, u32x4 (&A)[NC]) {
    const int off = (j < ntile ? (u_o * p.d_o + j) * FRAG : kOob) + alane;
#pragma unroll
    for (int c = 0; c < NC; ++c) A[c] = __builtin_amdgcn_raw_buffer_load_b128(rw, off, c * (2 * TM * 16), 0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto compute = [&](int s, const u32x4 (&A)[NC]) {
    const unsigned char *src = lds + (s & 1) * BUF;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const unsigned char *bsrc = src + ((2 * c + h2) * kCW) * 16;   // (block parity = h2: the swizzle is per lane)
      const u32x4 B0 = *reinterpret_cast<const u32x4 *>(bsrc + boff0);
      const u32x4 B1 = *reinterpret_cast<const u32x4 *>(bsrc + boff1);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[c]), __builtin_bit_cast(bf16x8, B0),
                                                        acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[c]), __builtin_bit_cast(bf16x8, B1),
                                                        acc[1], 0, 0, 0);
    }
  };
  u32x4 W0[NC], W1[NC];
  issue_weights(0, W0);
  __syncthreads();          // stage 0 is in LDS
  int done = 0;             // stages whose closing barrier this wave has passed
  auto cstep = [&](int j, const u32x4 (&cur)[NC], u32x4 (&nxt)[NC]) {
    const int s = table(p.max_stages + wid * p.d_o + j);
    for (; done < s; ++done) __syncthreads();   // stages of tile columns this tile row lacks
    issue_weights(j + 1, nxt);
    compute(s, cur);
    __syncthreads();
    ++done;
  };
  for (int j = 0; j < ntile; j += 2) {
    cstep(j, W0, W1);
    if (j + 1 < ntile) cstep(j + 1, W1, W0);
  }
  for (; done < cnt; ++done) __syncthreads();

  // Epilogue.  32x32 accumulator: register r of lane (n32, h2) is row 8 * (r / 4) + 4 * h2 + r % 4,
  // column n32 of the block.
  if (ntile == 0) return;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t n = n0 + 32 * h + n32;
    if (n >= out_n) continue;
    const int64_t m0 = int64_t(u_o) * TM + 4 * h2;
    if (out_bf16) {
      uint16_t *o = reinterpret_cast<uint16_t *>(out) + m0 * out_ld + n;
#pragma unroll
      for (int r = 0; r < 16; ++r) o[(8 * (r >> 2) + (r & 3)) * out_ld] = uint16_t(bf16_bits(acc[h][r]));
    } else {
      float *o = reinterpret_cast<float *>(out) + m0 * out_ld + n;
#pragma unroll
      for (int r = 0; r < 16; ++r) o[(8 * (r >> 2) + (r & 3)) * out_ld] = acc[h][r];
    }
  }
}

typedef void (*tile_fn)(TileParams);
struct TileEntry {
  int NC;
  tile_fn fn;
  int lds_set;   // largest dynamic LDS size requested for fn so far
};
TileEntry kTileTable[] = {{2, spmm_tile_bf16<2>, 0},   {4, spmm_tile_bf16<4>, 0},   {5, spmm_tile_bf16<5>, 0},
                          {8, spmm_tile_bf16<8>, 0},   {9, spmm_tile_bf16<9>, 0},   {16, spmm_tile_bf16<16>, 0},
                          {18, spmm_tile_bf16<18>, 0}, {20, spmm_tile_bf16<20>, 0}};

struct TileState {
  int32_t *stages = nullptr, *counts = nullptr;
  int max_stages = 0, RG = 0;
  std::vector<int32_t> host_table;   // stages then counts: what the kernel arguments carry when it is short enough
  int32_t *colbase = nullptr;        // fused convolution: pixel offsets of the column octets for the geometry below
  int64_t conv_key[3] = {0, 0, 0};   // images, height, width
};

#define RBGP_HIP(call)                                                              \
  do {                                                                              \
    hipError_t e_ = (call);                                                         \
    if (e_ != hipSuccess) {                                                         \
      char buf_[256];                                                               \
      std::snprintf(buf_, sizeof buf_, "%s: %s", #call, hipGetErrorString(e_));     \
      rbgp_set_hip_error(buf_);                                                     \
      return RBGP_EHIP;                                                             \
    }                                                                               \
  } while (0)

int build_state(const rbgp_mask *m, TileState *st) {
  const int a_o = m->a[0], d_o = m->d[0], c_o = m->c[0];
  const int RG = (a_o + 3) / 4;
  // stage list of a row group: the tile columns that any of its four tile rows has, ascending
  std::vector<std::vector<int32_t>> cols(static_cast<size_t>(RG));
  int max_stages = 1;
  for (int rg = 0; rg < RG; ++rg) {
    std::vector<char> has(static_cast<size_t>(c_o), 0);
    for (int u = rg * 4; u < std::min(a_o, rg * 4 + 4); ++u)
      for (int j = 0; j < d_o; ++j) has[size_t(m->adj[0][size_t(u) * d_o + j])] = 1;
    for (int v = 0; v < c_o; ++v)
      if (has[size_t(v)]) cols[size_t(rg)].push_back(v);
    max_stages = std::max(max_stages, int(cols[size_t(rg)].size()));
  }
  const int rec = max_stages + 4 * d_o;
  std::vector<int32_t> stages(size_t(RG) * rec, 0), counts(static_cast<size_t>(RG), 0);
  for (int rg = 0; rg < RG; ++rg) {
    const std::vector<int32_t> &cl = cols[size_t(rg)];
    int32_t *out = stages.data() + size_t(rg) * rec;
    std::copy(cl.begin(), cl.end(), out);
    counts[size_t(rg)] = int32_t(cl.size());
    for (int w = 0; w < 4; ++w) {
      const int u = rg * 4 + w;
      for (int j = 0; j < d_o && u < a_o; ++j) {
        const int32_t v = m->adj[0][size_t(u) * d_o + j];
        out[max_stages + w * d_o + j] = int32_t(std::lower_bound(cl.begin(), cl.end(), v) - cl.begin());
      }
    }
  }
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(&st->stages), stages.size() * 4));
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(&st->counts), counts.size() * 4));
  RBGP_HIP(hipMemcpy(st->stages, stages.data(), stages.size() * 4, hipMemcpyHostToDevice));
  RBGP_HIP(hipMemcpy(st->counts, counts.data(), counts.size() * 4, hipMemcpyHostToDevice));
  st->max_stages = max_stages;
  st->RG = RG;
  st->host_table = stages;
  st->host_table.insert(st->host_table.end(), counts.begin(), counts.end());
  return RBGP_OK;
}

}  // namespace

void rbgp_tile_release(void *state) {
  TileState *st = static_cast<TileState *>(state);
  if (!st) return;
  if (st->stages) (void)hipFree(st->stages);
  if (st->counts) (void)hipFree(st->counts);
  if (st->colbase) (void)hipFree(st->colbase);
  delete st;
}

int rbgp_tile_launch(const rbgp_mask *m, void **state, bool out_bf16, int64_t N, const void *packed, const void *I,
                     int64_t ldI, void *O, int64_t ldO, void *stream, const rbgp_conv_geometry *conv) {
  const rbgp_tile_plan pl = rbgp_plan_tile(m);
  if (!pl.ok) return RBGP_EUNSUPPORTED;
  int64_t chan_bytes = 0, x_bytes = 0;
  if (conv) {
    // the nine taps are the columns of a complete G_b; a lane's eight columns are eight pixels of one image row
    if (m->c[3] != 9 || m->d[3] != 9) return RBGP_EUNSUPPORTED;
    if (conv->images <= 0 || conv->height <= 0 || conv->width <= 0 || conv->width % 8) return RBGP_ESHAPE;
    if (N != conv->images * conv->height * conv->width) return RBGP_ESHAPE;
    if (reinterpret_cast<uintptr_t>(I) % 4) return RBGP_ESHAPE;
    chan_bytes = conv->images * (conv->height + 2) * (conv->width + 2) * 2;
    x_bytes = (m->K / 9) * chan_bytes;
    if (x_bytes + 64 >= (int64_t(1) << 30)) return RBGP_EUNSUPPORTED;   // 32-bit offsets, below the idle slots' offset
    ldI = 8;   // (unused by the kernel)
  } else {
    if ((reinterpret_cast<uintptr_t>(I) & 15) || (ldI % 8)) return RBGP_ESHAPE;
    // 32-bit offsets address the rows of one stage (and stay below the out-of-range offset of idle load slots)
    if (int64_t(pl.TKP) * ldI * 2 + 256 >= (int64_t(1) << 30)) return RBGP_EUNSUPPORTED;
  }
  TileState *st = static_cast<TileState *>(*state);
  if (!st) {
    st = new (std::nothrow) TileState();
    if (!st) return RBGP_ENOMEM;
    *state = st;
  }
  if (!st->stages) {
    int rc = build_state(m, st);
    if (rc) return rc;
  }
  TileParams p;
  p.Wp = packed; p.I = I; p.O = O;
  p.stages = st->stages; p.counts = st->counts;
  p.N = N; p.ldI = ldI; p.ldO = ldO; p.K = m->K;
  p.obf16 = out_bf16 ? 1 : 0;
  p.max_stages = st->max_stages;
  p.a_o = m->a[0]; p.d_o = m->d[0];
  p.TK = pl.TK;
  p.inl_ok = int(st->host_table.size()) <= kInline;
  p.tab_bytes = p.inl_ok ? 0 : ((st->max_stages + 4 * m->d[0]) * 4 + 15) / 16 * 16;
  if (p.inl_ok) std::copy(st->host_table.begin(), st->host_table.end(), p.inl);
  const int64_t ntiles = (N + kCW - 1) / kCW;
  p.ntiles = int(ntiles); p.RG = st->RG;
  p.conv = conv ? 1 : 0;
  p.conv_w2 = conv ? int(conv->width + 2) : 0;
  p.chan_bytes = uint32_t(chan_bytes);
  p.x_bytes = x_bytes;
  p.colbase = nullptr;
  if (conv) {
    int64_t *key = st->conv_key;
    if (st->colbase && (key[0] != conv->images || key[1] != conv->height || key[2] != conv->width)) {
      (void)hipFree(st->colbase);   // (waits for launches that still read the old table)
      st->colbase = nullptr;
    }
    if (!st->colbase) {
      // padding octets of the last tile point at the first pixel: their columns are never stored
      const int64_t H = conv->height, W = conv->width;
      std::vector<int32_t> cb(size_t(ntiles) * 8, int32_t((W + 3) * 2));
      for (int64_t n = 0; n < N; n += 8) {
        const int64_t img = n / (H * W), y = (n % (H * W)) / W, x = n % W;
        cb[size_t(n / 8)] = int32_t(((img * (H + 2) + y + 1) * (W + 2) + x + 1) * 2);
      }
      RBGP_HIP(hipMalloc(reinterpret_cast<void **>(&st->colbase), cb.size() * 4));
      RBGP_HIP(hipMemcpy(st->colbase, cb.data(), cb.size() * 4, hipMemcpyHostToDevice));
      key[0] = conv->images; key[1] = conv->height; key[2] = conv->width;
    }
    p.colbase = st->colbase;
  }
  p.w_bytes = uint32_t(pl.packed_elems * 2);
  p.n_round_bytes = uint32_t((N + 7) / 8 * 8 * 2);
  const int64_t blocks = 8 * ((ntiles + 7) / 8) * st->RG;
  if (blocks > 0x7fffffff || N * 2 + 16 >= (int64_t(1) << 32)) return RBGP_EUNSUPPORTED;
  TileEntry *te = nullptr;
  for (TileEntry &e : kTileTable)
    if (e.NC * 16 == pl.TKP) te = &e;
  if (!te) return RBGP_EUNSUPPORTED;
  const tile_fn fn = te->fn;
  const size_t lds = size_t(p.tab_bytes) + size_t(2) * (pl.TKP / 8) * kCW * 16;
  if (lds > 160 * 1024) return RBGP_EUNSUPPORTED;
  // (the attribute call costs microseconds on the host: once per kernel and size, not per launch; a racing
  // second thread at worst repeats the call)
  if (lds > 64 * 1024 && int(lds) > te->lds_set) {
    RBGP_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)));
    te->lds_set = int(lds);
  }
  hipLaunchKernelGGL(fn, dim3(unsigned(blocks)), dim3(512), lds, static_cast<hipStream_t>(stream), p);
  RBGP_HIP(hipGetLastError());
  return RBGP_OK;
}
