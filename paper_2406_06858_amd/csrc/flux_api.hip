// Host side of the library: argument validation, TileCoord tables, the AllGather copy driver
// (paper Alg. 3, pull form), the non-overlapped baseline and the C ABI declared in flux.h.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstring>
#include <vector>

#include "flux_internal.h"

namespace flux {

// (not const: a const table of host function pointers would also be emitted for the device)
CfgInfo g_cfgs[NUM_CFGS] = {
    {256, 256, 64, 1, 2, launch_cfg1}, {256, 128, 64, 1, 3, launch_cfg2}, {128, 128, 64, 2, 2, launch_cfg3},
    {64, 64, 64, 2, 2, launch_cfg4},   {64, 128, 64, 2, 2, launch_cfg5},  {32, 128, 64, 2, 2, launch_cfg6},
    {64, 64, 64, 1, 6, launch_cfg7},   {32, 128, 64, 1, 6, launch_cfg8},  {64, 128, 64, 1, 4, launch_cfg9},
    {64, 128, 64, 2, 3, launch_cfg10},
};

constexpr int N_CU = 256;                      // compute units of an MI355X
constexpr int N_XCD = 8;                       // accelerator dies of an MI355X, one L2 each
constexpr unsigned long long DEFAULT_TIMEOUT_TICKS = 1000000000ull;   // 10 s at 100 MHz

static thread_local int g_last_hip_error = 0;
static thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;
static thread_local flux_trace_record_t* g_trace_buf = nullptr;
static thread_local size_t g_trace_bytes = 0;

#define FLUX_HIP(expr)                                  \
  do {                                                  \
    hipError_t e__ = (expr);                            \
    if (e__ != hipSuccess) {                            \
      g_last_hip_error = (int)e__;                      \
      (void)hipGetLastError();                          \
      return FLUX_ERR_HIP;                              \
    }                                                   \
  } while (0)

// ------------------------------------------------------------------------------------------
// small kernels
// ------------------------------------------------------------------------------------------

// Puts the signal array in its preset state (local communication tiles 1, the others 0;
// paper Sec. 4.3 "Signals") and optionally clears the workspace header.
__global__ void preset_kernel(uint32_t* signals, int n_signals, int local_lo, int local_hi,
                              uint32_t* header, int header_words) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (signals != nullptr && i < n_signals) signals[i] = (i >= local_lo && i < local_hi) ? 1u : 0u;
  if (header != nullptr && i < header_words) header[i] = 0u;
}

struct CopyArgs {
  const uint4* src[FLUX_MAX_RANKS];   // chunk sources, indexed by rank
  uint4* dst;                         // A_agg
  int32_t order[FLUX_MAX_RANKS];      // chunks to move, in transfer order
  int32_t n_order;
  int32_t tiles_per_chunk;            // communication tiles per chunk
  unsigned long long tile_vec;        // 16-byte vectors per communication tile
  uint32_t* signals;                  // may be null (baseline copy: nothing to claim, count or signal)
  uint32_t* counters;
  uint32_t* claims;                   // [signals][pieces]
  int pieces;                         // pieces per communication tile; workgroup w takes w, w + gridDim.x, ...
  uint32_t call_id;
  uint32_t* started;                  // may be null
  unsigned long long pace_ticks;      // 100 MHz ticks per communication tile, 0 = unpaced
  AggPitch pitch;                     // rows of the gathered matrix: vectors in one, vectors from one to the next
  int32_t rows_per_tile;
};

// Copy driver as one kernel: all workgroups move communication tile after communication tile
// in transfer order (DataTransfer of Alg. 3), workgroup w taking pieces w, w + gridDim.x, ... of each
// unless a waiting GEMM workgroup got to a piece first; whoever finishes a tile's last piece sets
// its signal (SetSignal).  A tile has more pieces than the driver has workgroups, so that many
// waiting workgroups can share one tile.  The data is stored write-through and each wave waits for its stores to be
// acknowledged before the workgroup counts itself in, so no cache write-back fence (which would
// sweep the whole L2 of the die, per tile) is needed to publish a tile.
__global__ void __launch_bounds__(256) ag_copy_kernel(const CopyArgs c) {
  __shared__ int mine;
  // The driver's waves share compute units with GEMM waves whose MFMAs are always ready to issue;
  // at equal priority the few memory instructions here would wait behind them.
  __builtin_amdgcn_s_setprio(3);
  const int n_tiles = c.n_order * c.tiles_per_chunk;
  if (c.started != nullptr && threadIdx.x == 0)
    __hip_atomic_fetch_add(c.started, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long t_start = wall_clock64();
  for (int idx = 0; idx < n_tiles; ++idx) {
    const int chunk = c.order[idx / c.tiles_per_chunk];
    const int t = idx % c.tiles_per_chunk;
    const int flag = chunk * c.tiles_per_chunk + t;
    const uint4* src = c.src[chunk] + (unsigned long long)t * c.tile_vec;
    uint4* dst = c.dst + (unsigned long long)flag * c.rows_per_tile * c.pitch.pitch_v;
    int moved = 0;
    for (int piece = (int)blockIdx.x; piece < c.pieces; piece += (int)gridDim.x) {
      if (c.signals != nullptr) {
        if (threadIdx.x == 0) mine = claim_piece(c.claims + (size_t)flag * c.pieces + piece, c.call_id) ? 1 : 0;
        __syncthreads();
        const bool take = mine != 0;
        __syncthreads();
        if (!take) continue;
      }
      copy_piece(src, dst, c.tile_vec, piece, c.pieces, (int)threadIdx.x, c.pitch);
      ++moved;
    }
    if (moved == 0) continue;
    // link emulation: the tile "arrives" no earlier than a link of the given rate allows
    // (its data may move while the link is still busy with the tile before)
    if (c.pace_ticks != 0 && threadIdx.x == 0)
      while (wall_clock64() - t_start < (unsigned long long)(idx + 1) * c.pace_ticks) __builtin_amdgcn_s_sleep(8);
    if (c.signals != nullptr) finish_pieces(c.counters + flag, c.signals + flag, c.pieces, moved);
  }
}

struct ReduceArgs {
  const void* C;                      // [M,N] out dtype
  const void* peers[FLUX_MAX_RANKS];
  void* outs[FLUX_MAX_RANKS];
  int32_t M, N, R, rank, S, partial_f32, out_f32;
  int32_t c_f32;                      // dtype of C
  int32_t row0, rows;                 // rows [row0, row0 + rows) of the [M,N] matrices
  int32_t ld_c, ld_peer, ld_out;      // row pitches in elements
};

// Baseline reduce-scatter: out[r] = C + sum of peer partials, 8 columns per thread.
__global__ void __launch_bounds__(256) rs_reduce_kernel(const ReduceArgs a) {
  const long long nvec = (long long)a.rows * a.N / 8;
  const int nv_row = a.N / 8;
  for (long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += (long long)gridDim.x * blockDim.x) {
    const int gm = a.row0 + (int)(v / nv_row);
    const int gn = (int)(v % nv_row) * 8;
    const size_t off = (size_t)gm * a.ld_c + gn, off_peer = (size_t)gm * a.ld_peer + gn;
    float x[8];
    if (a.c_f32) {
      const float* p = static_cast<const float*>(a.C) + off;
      const uint4 u = ld_stream16(p), w = ld_stream16(p + 4);
      x[0] = __uint_as_float(u.x); x[1] = __uint_as_float(u.y); x[2] = __uint_as_float(u.z); x[3] = __uint_as_float(u.w);
      x[4] = __uint_as_float(w.x); x[5] = __uint_as_float(w.y); x[6] = __uint_as_float(w.z); x[7] = __uint_as_float(w.w);
    } else {
      const uint4 w = ld_stream16(static_cast<const __bf16*>(a.C) + off);
      x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
      x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
    }
    for (int j = 0; j < a.R; ++j) {
      if (j == a.rank) continue;
      if (a.partial_f32) {
        const float* p = static_cast<const float*>(a.peers[j]) + off_peer;
        const uint4 u = ld_stream16(p), w = ld_stream16(p + 4);
        x[0] += __uint_as_float(u.x); x[1] += __uint_as_float(u.y); x[2] += __uint_as_float(u.z); x[3] += __uint_as_float(u.w);
        x[4] += __uint_as_float(w.x); x[5] += __uint_as_float(w.y); x[6] += __uint_as_float(w.z); x[7] += __uint_as_float(w.w);
      } else {
        const uint4 w = ld_stream16(static_cast<const __bf16*>(a.peers[j]) + off_peer);
        x[0] += bf16_lo(w.x); x[1] += bf16_hi(w.x); x[2] += bf16_lo(w.y); x[3] += bf16_hi(w.y);
        x[4] += bf16_lo(w.z); x[5] += bf16_hi(w.z); x[6] += bf16_lo(w.w); x[7] += bf16_hi(w.w);
      }
    }
    const int r = gm / a.S;
    const size_t o = (size_t)(gm - r * a.S) * a.ld_out + gn;
    if (a.out_f32) {
      float* q = static_cast<float*>(a.outs[r]) + o;
      st_stream16(q, make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])));
      st_stream16(q + 4, make_uint4(__float_as_uint(x[4]), __float_as_uint(x[5]), __float_as_uint(x[6]), __float_as_uint(x[7])));
    } else {
      uint4 w;
      w.x = pack_bf16x2(x[0], x[1]); w.y = pack_bf16x2(x[2], x[3]);
      w.z = pack_bf16x2(x[4], x[5]); w.w = pack_bf16x2(x[6], x[7]);
      st_stream16(static_cast<__bf16*>(a.outs[r]) + o, w);
    }
  }
}

struct ReadyReduceArgs {
  const void* staged[FLUX_MAX_RANKS];   // [S,N] partials for this slice, one per producer, in rank order
  void* out;                            // [S,N]
  uint32_t* tile_ready;                 // [tiles_m * tiles_n] of the whole [M,N] grid
  uint32_t* status;                     // status block (code, detail)
  unsigned long long timeout_ticks;
  int32_t S, N, R, partial_f32, out_f32;
  int32_t ld;                           // row pitch of the staged matrices and of out, in elements
  int32_t bm, bn, tiles_n;              // the producers' tile shape
  int32_t row0;                         // first global row of the slice
  int32_t mt_lo, n_mt;                  // m-tiles that overlap the slice
  int32_t producers;                    // counter value that means "every producer has written the tile"
};

// Consumer side of the tile-ready handshake (Sec. 4.2, "Reduce", second form: a reducer on the
// destination that takes tiles as they come up).  A few persistent workgroups walk over the tiles
// that overlap this rank's slice; for each, one lane polls the tile's counter (bounded), then the
// workgroup sums the producers' staged rows of that tile in rank order, fp32, and writes the slice.
// Staged data is read at device scope (past this die's L2): the producers wrote it through.
__global__ void __launch_bounds__(256) rs_ready_reduce_kernel(const ReadyReduceArgs a) {
  __shared__ int outcome;
  const int n_tiles = a.n_mt * a.tiles_n;
  const int elem = a.partial_f32 ? 4 : 2;
  constexpr int SC1 = 16;                                     // cache-policy bit: device scope
  for (int t = (int)blockIdx.x; t < n_tiles; t += (int)gridDim.x) {
    const int mt = a.mt_lo + t / a.tiles_n, nt = t % a.tiles_n;
    if (threadIdx.x == 0) {
      const uint32_t* c = a.tile_ready + (size_t)mt * a.tiles_n + nt;
      const unsigned long long t0 = wall_clock64();
      int ok = 1;
      while (__hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) < (uint32_t)a.producers) {
        if (wall_clock64() - t0 > a.timeout_ticks) {
          if (atomicCAS(a.status, 0u, (uint32_t)FLUX_ERR_TIMEOUT) == 0u) a.status[1] = (uint32_t)(mt * a.tiles_n + nt);
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(32);
      }
      outcome = ok;
    }
    __syncthreads();
    const int ok = outcome;
    __syncthreads();                    // everyone has read it before thread 0 writes the next one
    if (!ok) continue;                  // the tile stays unwritten; the status block says which
    // rows of the tile that belong to this slice, as local rows
    const int g0 = mt * a.bm > a.row0 ? mt * a.bm : a.row0;
    const int g1 = (mt + 1) * a.bm < a.row0 + a.S ? (mt + 1) * a.bm : a.row0 + a.S;
    const int c0 = nt * a.bn, c1 = c0 + a.bn < a.N ? c0 + a.bn : a.N;
    const int vec_per_row = (c1 - c0) / 8;
    const int nvec = (g1 - g0) * vec_per_row;
    // the staged matrices through buffer resources based at the first row of the tile within the
    // slice (uniform; a lane's offset from there stays below 256 rows * pitch * 4 bytes < 2^31)
    const size_t tile_base = (size_t)(g0 - a.row0) * a.ld;
    for (int v = (int)threadIdx.x; v < nvec; v += (int)blockDim.x) {
      const int tr = v / vec_per_row, col = c0 + (v % vec_per_row) * 8;
      const size_t o = tile_base + (size_t)tr * a.ld + col;
      const int voff = (int)(((uint32_t)tr * (uint32_t)a.ld + (uint32_t)col) * (uint32_t)elem);
      float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int j = 0; j < a.R; ++j) {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned char*>(static_cast<const unsigned char*>(a.staged[j])) + tile_base * elem, 0, 0x7fffffff, 0x00027000);
        if (a.partial_f32) {
          const u32x4 u = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, 0, SC1), w = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 16, 0, SC1);
#pragma unroll
          for (int e = 0; e < 4; ++e) { x[e] += __uint_as_float(u[e]); x[4 + e] += __uint_as_float(w[e]); }
        } else {
          const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, 0, SC1);
#pragma unroll
          for (int e = 0; e < 4; ++e) { x[2 * e] += bf16_lo(w[e]); x[2 * e + 1] += bf16_hi(w[e]); }
        }
      }
      if (a.out_f32) {
        float* q = static_cast<float*>(a.out) + o;
        st_stream16(q, make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])));
        st_stream16(q + 4, make_uint4(__float_as_uint(x[4]), __float_as_uint(x[5]), __float_as_uint(x[6]), __float_as_uint(x[7])));
      } else {
        uint4 w;
        w.x = pack_bf16x2(x[0], x[1]); w.y = pack_bf16x2(x[2], x[3]);
        w.z = pack_bf16x2(x[4], x[5]); w.w = pack_bf16x2(x[6], x[7]);
        st_stream16(static_cast<__bf16*>(a.out) + o, w);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// planning
// ------------------------------------------------------------------------------------------

struct Plan {
  int cfg;          // index into g_cfgs
  int bm, bn, bk;
  int tiles_m, tiles_n;
  int split_k, k_per_split;
  int full_tiles, split_tiles;   // tiles computed whole / tiles cut along K (the last ones in TileCoord order)
  int edge;
  int n_xcd;
  int ctpc;         // communication tiles per chunk
  // AllGather copy driver
  int copy_wgs;             // workgroups of the copy kernel
  int copy_pieces;          // pieces per communication tile (the unit a workgroup claims and moves)
  int copy_help;            // waiting GEMM workgroups may take pieces
  int copy_self;            // no copy kernel at all: the GEMM grid moves everything
  int copy_owners;          // ... its first copy_owners workgroups sharing the pieces out by index
  int defer_tiles;          // ... the last defer_tiles remote communication tiles carried inside the first round's main loops,
  int defer_steps;          //     defer_steps vectors per thread and tile
  unsigned long long pace_ticks;   // ... counted in on a link's schedule (100 MHz ticks per communication tile; 0: as they come)
  int resident;             // reduce-scatter: one resident workgroup per compute unit walks the blocks ...
  uint32_t resident_delay_ticks;   // ... every second group of eight starting this late (100 MHz ticks)
  size_t claim_bytes;       // claim words in the workspace, after the header
};

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Row pitches in elements (0 in the problem: packed).
static inline long long pitch_a(const flux_problem_t* p) { return p->lda ? p->lda : p->K; }
static inline long long pitch_b(const flux_problem_t* p) { return p->ldb ? p->ldb : (p->b_is_nk ? p->K : p->N); }
static inline long long pitch_c(const flux_problem_t* p) { return p->ldc ? p->ldc : p->N; }

static int validate_problem(int op, const flux_problem_t* p) {
  if (p == nullptr) return FLUX_ERR_INVALID_ARG;
  if (op != FLUX_OP_RS && op != FLUX_OP_AG) return FLUX_ERR_INVALID_ARG;
  if (p->M <= 0 || p->N <= 0 || p->K <= 0) return FLUX_ERR_SHAPE;
  if (p->R < 1 || p->R > FLUX_MAX_RANKS) return FLUX_ERR_SHAPE;
  if (p->rank < 0 || p->rank >= p->R) return FLUX_ERR_INVALID_ARG;
  if (p->M % p->R != 0 || p->N % 8 != 0 || p->K % 8 != 0) return FLUX_ERR_SHAPE;
  // every matrix stays below 2^31 elements: the kernels address operands through 32-bit buffer offsets
  if ((long long)p->M * p->N >= (1ll << 31) || (long long)p->M * p->K >= (1ll << 31) ||
      (long long)p->K * p->N >= (1ll << 31)) return FLUX_ERR_SHAPE;
  // row pitches: at least a row, rows stay 16-byte aligned, and the last element's index stays below 2^31 too
  if (p->lda < 0 || p->ldb < 0 || p->ldc < 0 || (p->b_is_nk != 0 && p->b_is_nk != 1) || p->reserved2 != 0) return FLUX_ERR_INVALID_ARG;
  const long long b_rows = p->b_is_nk ? p->N : p->K, b_cols = p->b_is_nk ? p->K : p->N;      // B as it lies in memory
  if (pitch_a(p) < p->K || pitch_b(p) < b_cols || pitch_c(p) < p->N) return FLUX_ERR_SHAPE;
  if (pitch_a(p) % 8 != 0 || pitch_b(p) % 8 != 0 || pitch_c(p) % 8 != 0) return FLUX_ERR_SHAPE;
  if ((long long)(p->M - 1) * pitch_a(p) + p->K >= (1ll << 31) || (b_rows - 1) * pitch_b(p) + b_cols >= (1ll << 31) ||
      (long long)(p->M - 1) * pitch_c(p) + p->N >= (1ll << 31)) return FLUX_ERR_SHAPE;
  // the reduce-scatter epilogue addresses a tile of fp32 partials (up to 256 rows) through a signed
  // 31-bit offset from the tile's origin: 256 rows of 4-byte elements must stay below 2^31 bytes
  if (p->N >= FLUX_MAX_N || pitch_c(p) >= FLUX_MAX_N) return FLUX_ERR_SHAPE;
  if (p->out_dtype != FLUX_BF16 && p->out_dtype != FLUX_F32) return FLUX_ERR_INVALID_ARG;
  if (op == FLUX_OP_RS && p->partial_dtype != FLUX_BF16 && p->partial_dtype != FLUX_F32) return FLUX_ERR_INVALID_ARG;
  if (p->tile_config < 0 || p->tile_config > NUM_CFGS) return FLUX_ERR_INVALID_ARG;
  if (p->split_k < 0 || p->split_k > 64) return FLUX_ERR_INVALID_ARG;
  if (p->copy_workgroups < 0 || p->copy_workgroups > 4096) return FLUX_ERR_INVALID_ARG;
  if (p->link_gbps < 0 || p->reserved != 0) return FLUX_ERR_INVALID_ARG;
  if (op == FLUX_OP_AG) {
    const int ctpc = p->comm_tiles_per_chunk <= 0 ? 1 : p->comm_tiles_per_chunk;
    const int S = p->M / p->R;
    if (S % ctpc != 0) return FLUX_ERR_SHAPE;
    if ((long long)ctpc * p->R > MAX_COMM_TILES) return FLUX_ERR_UNSUPPORTED;
  }
  return FLUX_OK;
}

// How K is cut for configuration `cfg`: `split` parts for the last `split_tiles` tiles of the grid
// (all of them for a uniform split), none for the others.
static void plan_split(const flux_problem_t* p, int cfg, long long tiles, int kt, int* split_out, long long* split_tiles_out) {
  int split = p->split_k;
  const long long slots = (long long)N_CU * g_cfgs[cfg].occupancy;
  if (split <= 0) {
    split = 1;
    if (g_cfgs[cfg].stages > 2) {
      // deep pipeline, one workgroup per CU: as many K parts as still give a single round, each
      // long enough for the pipeline to fill
      if (tiles < slots) split = (int)std::max<long long>(1, std::min<long long>(slots / tiles, kt / 8));
    } else if (tiles < 256) {                   // too few tiles to fill the chip: cut K as well
      split = (int)std::min<long long>((512 + tiles - 1) / tiles, 16);
      split = std::max(1, std::min(split, kt / 4));
      // parked fp32 partials (written and re-read) should not outweigh the operands themselves
      const long long operands = (long long)p->M * p->K + (long long)p->K * p->N;
      const long long cap = operands / (4ll * p->M * p->N);
      split = (int)std::max<long long>(1, std::min<long long>(split, cap));
    }
  }
  long long split_tiles = tiles;
  if (p->split_k <= 0 && split == 1 && !(p->flags & FLUX_FLAG_NO_TAIL_SPLIT)) {
    // A grid of a few rounds whose last round fills at most half of the chip: cut only that
    // round's tiles along K so that it too occupies every CU, for a fraction of a round's time.
    const long long rem = tiles % slots;
    if (tiles > slots && tiles < 8 * slots && rem > 0 && 2 * rem <= slots) {
      const int ts = (int)std::min<long long>(std::min<long long>(slots / rem, 8), kt / 4);
      if (ts > 1) { split = ts; split_tiles = rem; }
    }
  }
  *split_out = std::max(1, std::min(split, kt));
  *split_tiles_out = split_tiles;
}

// Estimated time of the GEMM under configuration `cfg`, in arbitrary units: rounds of the grid
// over the chip's workgroup slots, times the tile's area, over the configuration's rate per slot
// (from measurements of full grids: 256x256 = 1, 256x128 on three stages 0.84, 128x128 two per
// CU 0.8 per CU; a ragged shape runs the register-staged kernel at about 0.7 of that).
static double plan_cost(const flux_problem_t* p, int cfg) {
  const int bm = g_cfgs[cfg].bm, bn = g_cfgs[cfg].bn, bk = g_cfgs[cfg].bk;
  const long long tiles = (long long)((p->M + bm - 1) / bm) * ((p->N + bn - 1) / bn);
  const int kt = (p->K + bk - 1) / bk;
  const long long slots = (long long)N_CU * g_cfgs[cfg].occupancy;
  int split;
  long long split_tiles;
  plan_split(p, cfg, tiles, kt, &split, &split_tiles);
  const double part = (1.0 + 0.04 * (split - 1)) / split;          // a K part, with its hand-over
  double rounds;
  if (split > 1 && split_tiles < tiles) rounds = (double)((tiles - split_tiles) / slots) + part * (double)((split_tiles * split + slots - 1) / slots);
  else rounds = part * (double)((tiles * split + slots - 1) / slots);
  double rate = cfg == 0 ? 1.0 : cfg == 1 ? 0.84 : 0.8 / g_cfgs[cfg].occupancy;
  if (p->M % bm != 0 || p->N % bn != 0 || p->K % bk != 0) rate *= 0.7;
  return rounds * (double)bm * (double)bn / rate;
}

static int make_plan(int op, const flux_problem_t* p, Plan* pl) {
  int st = validate_problem(op, p);
  if (st != FLUX_OK) return st;
  int cfg;
  if (p->tile_config > 0) {
    cfg = p->tile_config - 1;
  } else {
    // few rows: the tile is bound by memory, so take the deep load pipeline if the shape allows its
    // direct-to-LDS loads (whole tiles along N and K; M may be ragged), else the two-stage twin
    const bool deep_ok = p->K % 64 == 0;
    if (p->M <= 32) cfg = (deep_ok && p->N % 128 == 0) ? 7 : 5;          // 32x128
    else if (p->M == 64 && deep_ok && p->N % 128 == 0 && p->N / 128 <= N_CU &&
             std::min<long long>(N_CU / (p->N / 128), p->K / 64 / 8) <= 5) {
      // 64 rows over a large weight matrix: 64x128 tiles on four stages where at most five K parts
      // fill the chip (12288x6144: 37 against 45 us, 6144x12288: 36 against 47 us for 64x64 tiles,
      // whose grid leaves a quarter of the chip idle there; no difference on 8192x3584 and 8192x8192)
      cfg = 8;
    }
    else if (p->M <= 64) cfg = (deep_ok && p->N % 64 == 0 && p->M == 64) ? 6 : 4;   // 64x64 deep, else 64x128
    else if ((long long)p->M * p->N <= 256ll * 1024) cfg = 3;            // 64x64, small problems
    else if (p->M == 128 && deep_ok && p->N % 128 == 0 && p->K > 8192 && 2ll * (p->N / 128) <= N_CU / 2) {
      // Two m-tiles, a long K and few columns: the two-per-CU 64x128 tile, whose finer K cut fills
      // its 512 slots (6144x12288: 55 against 66 us for 64x128 on four stages, weights from HBM).
      // (64x64 tiles on six stages are 11-19 % ahead on 3584x8192 and 8192x3584 while the weights
      // are still in the Infinity Cache and 3-4 % behind when they come from HBM: not taken.)
      cfg = 9;
    }
    else if (p->M == 256 && deep_ok && p->N % 128 == 0 && p->K >= 6144 &&
             std::min<long long>(N_CU / (p->N / 128), p->K / 64 / 8) <= 5) {
      // One m-tile of 256 rows: 256x128 tiles read the weights once; they pay where filling the
      // chip takes at most five K parts (the workgroup that arrives last at a tile reads all parts
      // back, at what one CU can pull): 12288x6144 64-70 us against 93-96 us for 64x128, 6144x12288
      // 68-72 against 88-91 us.
      cfg = 1;
    }
    else if (p->M == 256 && deep_ok && p->N % 128 == 0 && p->K >= 8192 && 4ll * (p->N / 128) <= N_CU) {
      // ... and where that takes more parts, over a long K: 64x128 tiles, two workgroups per CU, K
      // cut so that every slot has a part (3584x8192, weights from HBM: 36-41 us against 40-44 us
      // for the same tile on four stages, one per CU).
      cfg = 9;
    }
    else if (p->M <= 256 && p->M % 64 == 0 && deep_ok && p->N % 128 == 0) cfg = 8;   // 64x128 deep
    else {
      // Large tiles: 256x256 moves the least operand data per flop but needs a grid that fills the
      // chip round by round; 256x128 and 128x128 give two and four times the tiles.  Take the one
      // with the least estimated time.  256x256 with a uniform K split is never worth it.
      cfg = 2;
      double best = plan_cost(p, 2);
      const double c1 = plan_cost(p, 1);
      if (c1 < best) { best = c1; cfg = 1; }
      if ((long long)((p->M + 255) / 256) * ((p->N + 255) / 256) >= 128) {
        const double c0 = plan_cost(p, 0);
        if (c0 <= best) { best = c0; cfg = 0; }
      }
    }
  }
  pl->cfg = cfg;
  pl->bm = g_cfgs[cfg].bm; pl->bn = g_cfgs[cfg].bn; pl->bk = g_cfgs[cfg].bk;
  pl->tiles_m = (p->M + pl->bm - 1) / pl->bm;
  pl->tiles_n = (p->N + pl->bn - 1) / pl->bn;
  if (pl->tiles_m > FLUX_MAX_M_TILES) return FLUX_ERR_UNSUPPORTED;
  const long long tiles = (long long)pl->tiles_m * pl->tiles_n;
  if (tiles > (1ll << 24)) return FLUX_ERR_UNSUPPORTED;
  const int kt = (p->K + pl->bk - 1) / pl->bk;
  int split;
  long long split_tiles;
  plan_split(p, cfg, tiles, kt, &split, &split_tiles);
  split = std::max(1, std::min(split, kt));
  const int kt_per = (kt + split - 1) / split;
  split = (kt + kt_per - 1) / kt_per;             // no empty splits
  if (split > 1 && split_tiles > MAX_SPLITK_TILES) return FLUX_ERR_UNSUPPORTED;
  pl->split_k = split;
  pl->k_per_split = kt_per * pl->bk;
  pl->split_tiles = split > 1 ? (int)split_tiles : (int)tiles;
  pl->full_tiles = (int)tiles - pl->split_tiles;
  // 0: the tile divides the shape; 1: ragged (register-staged kernel); 2: only M is ragged and the
  // configuration has the deep pipeline, which reads rows past M as zeros.  That relies on the
  // buffer range check, so it is only used where a lane's row is entirely part of its own offset
  // (32-row tiles: one load instruction per wave covers all rows), not added per instruction.
  if ((p->N % pl->bn != 0) || (p->K % pl->bk != 0)) pl->edge = 1;
  else if (p->M % pl->bm != 0) pl->edge = (g_cfgs[cfg].stages > 2 && pl->bm == 32) ? 2 : 1;   // (see below)
  else pl->edge = 0;
  pl->n_xcd = (p->flags & (FLUX_FLAG_NO_SWIZZLE | FLUX_FLAG_NO_XCD_REMAP)) ? 1 : N_XCD;
  // Reduce-scatter grids of many short tiles.  Workgroups that the hardware dispatches one per tile
  // run in lock step (a freed compute unit gets its next workgroup only when its turn comes in the
  // dispatch order), so all 256 epilogues pull their peers' tiles at the same time and share what
  // the memory delivers (44 us per 256x256 tile with 7 peers), and then all main loops run with the
  // memory idle.  A compute unit alone pulls more than its 1/256 share (32 us per tile).  So: one
  // resident workgroup per compute unit, walking the block sequence with the grid's stride, and
  // half of them starting half a period late, which puts one half's epilogues beside the other
  // half's main loops for the rest of the kernel (8192x12288x1536, 8 ranks: 447 against 500 us).
  // With a long K the main loops drift apart by themselves within a round or two and nothing is
  // gained (8192x12288x6144: 1114 us either way), and a grid of fewer than four rounds does not
  // earn the late start back.
  pl->resident = 0;
  pl->resident_delay_ticks = 0;
  if (op == FLUX_OP_RS && !(p->flags & (FLUX_FLAG_RS_WRITE_ONLY | FLUX_FLAG_RS_ATOMIC | FLUX_FLAG_NO_RESIDENT_GRID)) &&
      g_cfgs[cfg].stages == 2 && g_cfgs[cfg].occupancy == 1 && pl->edge == 0 &&
      (long long)pl->full_tiles + (long long)pl->split_tiles * pl->split_k >= 4ll * N_CU && p->K <= 3072) {
    pl->resident = 1;
    // half a period: (main loop + epilogue of a tile on a compute unit that shares the memory with
    // half of the others) / 2; 1.5 us per 64-deep K slab of a 256x256 tile, 33 GB/s per unit
    const double main_ticks = 150.0 * (double)kt;
    const double tile_bytes = (double)pl->bm * pl->bn *
        ((p->R - 1) * (p->partial_dtype == FLUX_F32 ? 4.0 : 2.0) + (p->out_dtype == FLUX_F32 ? 4.0 : 2.0));
    const double epi_ticks = tile_bytes / 33.0e9 * 1.0e8;
    pl->resident_delay_ticks = (uint32_t)std::min(20000.0, (main_ticks + epi_ticks) / 2);
  }
  pl->ctpc = p->comm_tiles_per_chunk <= 0 ? 1 : p->comm_tiles_per_chunk;
  pl->copy_wgs = 0; pl->copy_pieces = 0; pl->copy_help = 0; pl->copy_self = 0; pl->copy_owners = 0; pl->claim_bytes = 0; pl->defer_tiles = 0; pl->defer_steps = 0; pl->pace_ticks = 0;
  if (op == FLUX_OP_AG) {
    // Driver: one piece of every communication tile per workgroup.  A small driver: it keeps the
    // later chunks coming in the background while waiting GEMM workgroups pull what they need now;
    // a large one would sit on compute units the GEMM wants.
    // ... and one that stands for a link needs no more workgroups than move data at the link's rate
    // (about 40 GB/s each): every one of them holds a compute unit for the whole transfer.
    // A driver that stands for a link gets as many workgroups as move data at the link's rate and no
    // more, since each keeps GEMM workgroups off a compute unit for as long as the transfer lasts.  A
    // unit copies about 20 GB/s beside a running GEMM, with four waves or with sixteen (a driver of 12
    // workgroups of 1024 threads moved 170 GB/s, one of 28 of 256 threads 870 GB/s), so a 1 TB/s link
    // costs some fifty units: that is the price of standing in for a link with compute units.
    int wgs = p->copy_workgroups > 0 ? p->copy_workgroups
                                     : (p->link_gbps > 0 ? std::max(4, std::min(64, (p->link_gbps + 19) / 20)) : 32);
    wgs = std::min(wgs, MAX_COPY_PIECES);
    const unsigned long long tile_vec = (unsigned long long)(p->M / p->R) * p->K / 8 / pl->ctpc;
    wgs = (int)std::max<unsigned long long>(1, std::min<unsigned long long>(wgs, (tile_vec + 255) / 256));
    pl->copy_wgs = wgs;
    pl->copy_pieces = wgs;
    pl->copy_help = !(p->flags & FLUX_FLAG_COPY_MEMCPY);
    // Unless the driver stands for a link (link_gbps), or the caller asks for one (copy_workgroups,
    // FLUX_FLAG_COPY_MEMCPY), none is launched: the GEMM grid moves the data itself before it looks
    // at its signals.  A driver workgroup holds a compute unit that a GEMM workgroup cannot share
    // (it needs the whole register file) and pushes that unit's tiles back by its own lifetime, a
    // whole extra round where the grid divided evenly before; on a grid that leaves units free it
    // still costs a second stream's fork and join, and waiting workgroups spin beside it.
    pl->copy_self = pl->copy_help && p->link_gbps == 0 && p->copy_workgroups == 0;
    const long long grid = (long long)pl->full_tiles + (long long)pl->split_tiles * pl->split_k;
    const long long slots = (long long)N_CU * g_cfgs[cfg].occupancy;
    const long long whole_tiles = pl->split_k == 1 ? tiles : (long long)pl->full_tiles;
    // what the two-stage kernel's workgroups can carry themselves (see SideCopy)
    const bool can_carry = g_cfgs[cfg].stages == 2 && g_cfgs[cfg].occupancy == 1 && pl->edge == 0 &&
                           !(p->flags & (FLUX_FLAG_AG_ABSENT_OWNERS | FLUX_FLAG_AG_COPY_UPFRONT)) && tile_vec * 16ull < (1ull << 31) &&
                           pitch_a(p) == p->K;      // (a tile is one run of memory on both sides)
    if (pl->copy_help && p->link_gbps > 0 && p->copy_workgroups == 0 && can_carry && (p->R - 1) * pl->ctpc <= 32 && p->R > 1) {
      // A transfer that stands for a link, without a driver: a driver's workgroups would each hold a
      // compute unit for as long as the transfer lasts, which no link does.  Every remote tile is
      // carried by the first round's workgroups, piece w by workgroup w: while a workgroup waits for
      // its own signals it moves its pieces in batches, afterwards inside its main loop, and a tile
      // is counted in (its signal set) on the link's schedule.
      const long long owners = std::min<long long>(grid, slots);
      pl->copy_self = 1;
      pl->copy_wgs = 0;
      pl->copy_pieces = (int)std::max<unsigned long long>(1, std::min<unsigned long long>(std::min<long long>(MAX_COPY_PIECES, owners), tile_vec / 1024));
      pl->copy_owners = (int)owners;
      pl->defer_tiles = (p->R - 1) * pl->ctpc;
      pl->defer_steps = (int)((tile_vec + (unsigned long long)pl->copy_pieces * 256 - 1) / ((unsigned long long)pl->copy_pieces * 256));
      pl->pace_ticks = std::max<unsigned long long>(1, (unsigned long long)((double)tile_vec * 16.0 / (double)p->link_gbps / 10.0));
    } else if (pl->copy_self) {
      // the first workgroups of the grid, as many as surely run at once, own the pieces
      pl->copy_wgs = 0;
      // pieces of 16 KiB or more, as many as the claim table allows
      pl->copy_pieces = (int)std::max<unsigned long long>(1, std::min<unsigned long long>(MAX_COPY_PIECES, tile_vec / 1024));
      pl->copy_owners = (int)std::min<long long>(grid, slots);
      if (p->flags & FLUX_FLAG_AG_ABSENT_OWNERS) pl->copy_owners = (int)std::min<long long>(2 * grid, 1 << 20);
      // A grid of several rounds needs only the chunks of its first round's tiles before it can
      // start.  The others are carried inside the first round's main loops, two 16-byte vectors per
      // thread and K slab, where they cost neither matrix-core time nor a wait: workgroup w moves
      // piece w of each of them.  Asked of the two-stage kernel on shapes the tile divides, with one
      // signal per chunk and the swizzled order (a band of tiles per chunk), a first round of whole
      // tiles that covers every piece, and a K long enough for all of a workgroup's vectors.
      const int S = p->M / p->R;
      const long long band_sz = (S % pl->bm == 0) ? (long long)(S / pl->bm) * pl->tiles_n : 0;
      if (can_carry && !(p->flags & FLUX_FLAG_NO_SWIZZLE) && pl->ctpc == 1 && band_sz > 0 && grid > slots &&
          whole_tiles >= slots && pl->copy_pieces <= pl->copy_owners) {
        const long long bands_first = (slots + band_sz - 1) / band_sz;       // bands the first round touches, the local one included
        const long long deferred = (long long)p->R - bands_first;             // remote chunks nobody needs before the second round
        const long long steps = (long long)((tile_vec + (unsigned long long)pl->copy_pieces * 256 - 1) / ((unsigned long long)pl->copy_pieces * 256));
        if (deferred >= 1 && (deferred * steps + 1) / 2 + 8 <= kt) {
          pl->defer_tiles = (int)deferred;
          pl->defer_steps = (int)steps;
        }
      }
    }
    pl->claim_bytes = (((size_t)p->R * pl->ctpc * pl->copy_pieces * 4) + 255) / 256 * 256;
  }
  return FLUX_OK;
}

static void ring_order(int rank, int R, int* order) {
  for (int d = 1; d < R; ++d) order[d - 1] = (rank + d) % R;
}

static int check_arrival(const flux_problem_t* p, const int32_t* arrival, int* order) {
  if (arrival == nullptr) { ring_order(p->rank, p->R, order); return FLUX_OK; }
  bool seen[FLUX_MAX_RANKS] = {false};
  for (int i = 0; i < p->R - 1; ++i) {
    const int c = arrival[i];
    if (c < 0 || c >= p->R || c == p->rank || seen[c]) return FLUX_ERR_INVALID_ARG;
    seen[c] = true;
    order[i] = c;
  }
  return FLUX_OK;
}

// Order in which m-tiles are scheduled: every m-tile gets a key and tiles are sorted by
// (key, index).  ReduceScatter: key = position of the owner of the tile's first row in the
// ring that starts after the local rank and ends on it.  AllGather: key = latest position, in
// [local chunk, arrival order...], among the chunks the tile's rows touch.
static void pack_order(TileMap* tm) {
  tm->packed = tm->tiles_m <= 16;
  tm->pad_ = 0;
  tm->order4 = 0;
  if (tm->packed)
    for (int t = 0; t < tm->tiles_m; ++t) tm->order4 |= (uint64_t)tm->m_order[t] << (4 * t);
}

static void build_tile_map(int op, const flux_problem_t* p, const Plan& pl, const int* arrival, TileMap* tm) {
  tm->tiles_m = pl.tiles_m;
  tm->tiles_n = pl.tiles_n;
  tm->n_xcd = pl.n_xcd;
  const int S = p->M / p->R;
  if (p->flags & FLUX_FLAG_NO_SWIZZLE) {
    tm->band_h = 1;
    for (int t = 0; t < pl.tiles_m; ++t) tm->m_order[t] = (uint16_t)t;
    pack_order(tm);
    return;
  }
  // a band = the m-tiles that wait for the same signal (one communication tile, Sec. 4.3), if whole
  // tiles make up a communication tile; else the m-tiles of one slice / chunk; else one m-tile
  const int Sc = (op == FLUX_OP_AG && S % pl.ctpc == 0) ? S / pl.ctpc : S;
  tm->band_h = (Sc % pl.bm == 0) ? Sc / pl.bm : ((S % pl.bm == 0) ? S / pl.bm : 1);
  int pos[FLUX_MAX_RANKS];
  if (op == FLUX_OP_RS) {
    for (int d = 1; d < p->R; ++d) pos[(p->rank + d) % p->R] = d - 1;
    pos[p->rank] = p->R - 1;
  } else {
    pos[p->rank] = 0;
    for (int i = 0; i < p->R - 1; ++i) pos[arrival[i]] = i + 1;
  }
  std::vector<std::pair<int, int>> keyed(pl.tiles_m);
  for (int t = 0; t < pl.tiles_m; ++t) {
    const int r0 = t * pl.bm;
    const int r1 = std::min(p->M, r0 + pl.bm) - 1;
    int key;
    if (op == FLUX_OP_RS) {
      key = pos[r0 / S];
    } else {
      key = 0;
      for (int c = r0 / S; c <= r1 / S; ++c) key = std::max(key, pos[c]);
    }
    keyed[t] = {key, t};
  }
  std::sort(keyed.begin(), keyed.end());
  for (int t = 0; t < pl.tiles_m; ++t) tm->m_order[t] = (uint16_t)keyed[t].second;
  pack_order(tm);
}

static size_t workspace_need(const Plan& pl) {
  size_t need = WS_HEADER_BYTES + pl.claim_bytes;
  if (pl.split_k > 1)
    need += (size_t)pl.split_k * pl.split_tiles * pl.bm * pl.bn * sizeof(float);
  return need;
}

static int check_workspace(const Plan& pl, int op, const void* ws, size_t bytes) {
  const bool needed = op == FLUX_OP_AG || pl.split_k > 1;
  if (!needed) return FLUX_OK;
  if (ws == nullptr || bytes < workspace_need(pl)) return FLUX_ERR_WORKSPACE;
  if (!aligned16(ws)) return FLUX_ERR_INVALID_ARG;
  return FLUX_OK;
}

static void fill_common(GemmArgs* a, const flux_problem_t* p, const Plan& pl, void* ws) {
  std::memset(a, 0, sizeof(*a));
  a->M = p->M; a->N = p->N; a->K = p->K;
  a->R = p->R; a->rank = p->rank; a->S = p->M / p->R;
  a->lda = (int32_t)pitch_a(p); a->ldb = (int32_t)pitch_b(p); a->ldc = (int32_t)pitch_c(p);
  a->b_is_nk = p->b_is_nk;
  a->partial_f32 = p->partial_dtype == FLUX_F32;
  a->out_f32 = p->out_dtype == FLUX_F32;
  a->split_k = pl.split_k;
  a->k_per_split = pl.k_per_split;
  a->full_tiles = pl.full_tiles;
  a->split_tiles = pl.split_tiles;
  a->rows_per_signal = std::max(1, (p->M / p->R) / pl.ctpc);
  a->timeout_ticks = p->spin_timeout_ticks ? p->spin_timeout_ticks : DEFAULT_TIMEOUT_TICKS;
  if (ws != nullptr) {
    unsigned char* w = static_cast<unsigned char*>(ws);
    a->status = reinterpret_cast<uint32_t*>(w + WS_STATUS_OFF);
    a->done_counter = reinterpret_cast<uint32_t*>(w + WS_DONE_OFF);
    a->started_counter = reinterpret_cast<uint32_t*>(w + WS_STARTED_OFF);
    a->sk_counters = reinterpret_cast<uint32_t*>(w + WS_TILECNT_OFF);
    a->copy_claims = reinterpret_cast<uint32_t*>(w + WS_HEADER_BYTES);
    a->copy_counters = reinterpret_cast<uint32_t*>(w + WS_COUNTER_OFF);
    a->sk_partials = reinterpret_cast<float*>(w + WS_HEADER_BYTES + pl.claim_bytes);
  }
}

// A pending tile-trace request of this thread: checked (and consumed) before anything is enqueued.
static int take_trace(const Plan& pl, flux_trace_record_t** out) {
  *out = g_trace_buf;
  const size_t bytes = g_trace_bytes;
  g_trace_buf = nullptr;
  g_trace_bytes = 0;
  if (*out == nullptr) return FLUX_OK;
  const size_t grid = (size_t)pl.full_tiles + (size_t)pl.split_tiles * pl.split_k;
  if (bytes < grid * sizeof(flux_trace_record_t)) { *out = nullptr; return FLUX_ERR_WORKSPACE; }
  return FLUX_OK;
}

static int launch_gemm(const Plan& pl, int epi, int wait, const GemmArgs& a, hipStream_t s) {
  const int grid = pl.full_tiles + pl.split_tiles * pl.split_k;
  hipEvent_t e0 = g_prof_start, e1 = g_prof_stop;
  g_prof_start = g_prof_stop = nullptr;
  if (e0) FLUX_HIP(hipEventRecord(e0, s));
  if (pl.resident && epi == EPI_RS && !wait && a.write_only == 0) {
    GemmArgs b = a;
    b.persist_blocks = grid;
    b.persist_delay_ticks = pl.resident_delay_ticks;
    FLUX_HIP(g_cfgs[pl.cfg].launch(epi, wait, pl.edge, b, N_CU, s));
  } else {
    FLUX_HIP(g_cfgs[pl.cfg].launch(epi, wait, pl.edge, a, grid, s));
  }
  if (e1) FLUX_HIP(hipEventRecord(e1, s));
  return FLUX_OK;
}

// `fused`: the copy driver of a fused call (claims, counters, signals, pacing); otherwise a plain
// copy of the listed chunks.
static int launch_copy(const flux_problem_t* p, const Plan& pl, const void* const* chunks, void* A_agg,
                       const int* order, int n_order, bool fused, uint32_t* signals, void* ws, uint32_t call_id,
                       hipStream_t s) {
  if (n_order == 0) return FLUX_OK;
  CopyArgs c;
  std::memset(&c, 0, sizeof(c));
  const unsigned long long chunk_vec = (unsigned long long)(p->M / p->R) * p->K / 8;
  for (int r = 0; r < p->R; ++r) c.src[r] = static_cast<const uint4*>(chunks[r]);
  c.dst = static_cast<uint4*>(A_agg);
  for (int i = 0; i < n_order; ++i) c.order[i] = order[i];
  c.n_order = n_order;
  c.tiles_per_chunk = fused ? pl.ctpc : 1;
  c.tile_vec = chunk_vec / c.tiles_per_chunk;
  c.pitch = AggPitch{(uint32_t)p->K / 8u, (uint32_t)(pitch_a(p) / 8)};
  c.rows_per_tile = (p->M / p->R) / c.tiles_per_chunk;
  // bytes / (GB/s) = ns; 10 ns per tick.  The baseline's copy is paced like the fused call's driver:
  // an emulated link delivers no faster when nothing overlaps with it.
  c.pace_ticks = p->link_gbps > 0 ? (unsigned long long)((double)c.tile_vec * 16.0 / (double)p->link_gbps / 10.0) : 0ull;
  int wgs;
  if (fused) {
    unsigned char* w = static_cast<unsigned char*>(ws);
    c.signals = signals;
    c.counters = reinterpret_cast<uint32_t*>(w + WS_COUNTER_OFF);
    c.claims = reinterpret_cast<uint32_t*>(w + WS_HEADER_BYTES);
    c.call_id = call_id;
    c.started = reinterpret_cast<uint32_t*>(w + WS_STARTED_OFF);
    wgs = pl.copy_wgs;
    c.pieces = pl.copy_pieces;
  } else {
    wgs = p->copy_workgroups > 0 ? p->copy_workgroups : 1024;
    wgs = (int)std::max<unsigned long long>(1, std::min<unsigned long long>(wgs, (c.tile_vec + 255) / 256));
    c.pieces = wgs;
  }
  hipLaunchKernelGGL(ag_copy_kernel, dim3(wgs), dim3(256), 0, s, c);
  FLUX_HIP(hipGetLastError());
  return FLUX_OK;
}

static std::atomic<uint32_t> g_call_id{1};
static uint32_t next_call_id() {
  uint32_t id;
  do { id = g_call_id.fetch_add(1, std::memory_order_relaxed); } while (id == 0);   // 0 = "never claimed"
  return id;
}

// Fork/join and per-chunk events belong to the calling host thread: a wait enqueued on an event
// refers to the record that preceded it on that thread, so calls of one thread may share a set,
// while two threads recording the same event could order a stream after the wrong fork.
static thread_local hipEvent_t g_fork = nullptr, g_join = nullptr;

static int get_events(hipEvent_t* fork, hipEvent_t* join) {
  if (g_fork == nullptr) {
    FLUX_HIP(hipEventCreateWithFlags(&g_fork, hipEventDisableTiming));
    FLUX_HIP(hipEventCreateWithFlags(&g_join, hipEventDisableTiming));
  }
  *fork = g_fork;
  *join = g_join;
  return FLUX_OK;
}

static thread_local hipEvent_t g_chunk_events[FLUX_MAX_RANKS] = {nullptr};

static int get_chunk_events(hipEvent_t** events) {
  for (int i = 0; i < FLUX_MAX_RANKS; ++i)
    if (g_chunk_events[i] == nullptr) FLUX_HIP(hipEventCreateWithFlags(&g_chunk_events[i], hipEventDisableTiming));
  *events = g_chunk_events;
  return FLUX_OK;
}


int gemm_rs_planned(const flux_problem_t* p, const Plan& pl, const void* A, const void* B, const void* const* peer_partials,
                    void* const* out_slices, void* workspace, size_t workspace_bytes, void* stream, uint32_t* tile_ready = nullptr);

}  // namespace flux

// Scratch memory of flux_gemm_rs_static: one array per GPU the library's code object is loaded on,
// there until the process ends.  In host code the array's name only stands for the symbol; its
// address on the current device is looked up once per device and used from then on.
static __device__ __align__(256) unsigned char flux_static_scratch[FLUX_STATIC_SCRATCH_BYTES];

namespace flux {

constexpr int MAX_DEVICES = 64;
static std::atomic<void*> g_scratch_ptr[MAX_DEVICES];

static int static_scratch(void** out) {
  int dev = -1;
  FLUX_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return FLUX_ERR_UNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    FLUX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(flux_static_scratch)));   // the current device's copy
    if (p == nullptr) return FLUX_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);              // (a racing thread stores the same address)
  }
  *out = p;
  return FLUX_OK;
}

}  // namespace flux

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
using namespace flux;

extern "C" {

int flux_version(void) { return 1; }

int flux_last_hip_error(void) { return g_last_hip_error; }

int flux_trace_next_call(void* records, size_t bytes) {
  if (records != nullptr && (!aligned16(records) || bytes < sizeof(flux_trace_record_t))) return FLUX_ERR_INVALID_ARG;
  g_trace_buf = static_cast<flux_trace_record_t*>(records);
  g_trace_bytes = records ? bytes : 0;
  return FLUX_OK;
}

int flux_profile_next_gemm(void* start_event, void* stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr)) return FLUX_ERR_INVALID_ARG;
  g_prof_start = static_cast<hipEvent_t>(start_event);
  g_prof_stop = static_cast<hipEvent_t>(stop_event);
  return FLUX_OK;
}

const char* flux_status_string(int status) {
  switch (status) {
    case FLUX_OK: return "ok";
    case FLUX_ERR_INVALID_ARG: return "invalid argument";
    case FLUX_ERR_SHAPE: return "unsupported shape";
    case FLUX_ERR_UNSUPPORTED: return "unsupported request";
    case FLUX_ERR_WORKSPACE: return "workspace missing or too small";
    case FLUX_ERR_HIP: return "HIP runtime error";
    case FLUX_ERR_TIMEOUT: return "signal wait timed out";
    default: return "unknown status";
  }
}

int flux_tile_config_count(void) { return NUM_CFGS; }

int flux_tile_config_info(int32_t id, int32_t* tile_m, int32_t* tile_n, int32_t* tile_k) {
  if (id < 1 || id > NUM_CFGS || !tile_m || !tile_n || !tile_k) return FLUX_ERR_INVALID_ARG;
  *tile_m = g_cfgs[id - 1].bm; *tile_n = g_cfgs[id - 1].bn; *tile_k = g_cfgs[id - 1].bk;
  return FLUX_OK;
}

int flux_default_order(int32_t rank, int32_t R, int32_t* order) {
  if (R < 1 || R > FLUX_MAX_RANKS || rank < 0 || rank >= R || (R > 1 && order == nullptr)) return FLUX_ERR_INVALID_ARG;
  ring_order(rank, R, order);
  return FLUX_OK;
}

size_t flux_workspace_bytes(int op, const flux_problem_t* p) {
  Plan pl;
  if (make_plan(op, p, &pl) != FLUX_OK) return 0;
  if (op == FLUX_OP_RS && pl.split_k <= 1) return 0;
  return workspace_need(pl);
}

int flux_init_buffers(int op, const flux_problem_t* p, void* workspace, size_t workspace_bytes,
                      uint32_t* signals, void* stream) {
  Plan pl;
  int st = make_plan(op, p, &pl);
  if (st != FLUX_OK) return st;
  if (workspace != nullptr && (workspace_bytes < WS_HEADER_BYTES + pl.claim_bytes || !aligned16(workspace))) return FLUX_ERR_WORKSPACE;
  if (workspace == nullptr && signals == nullptr) return FLUX_OK;
  const int n_sig = (op == FLUX_OP_AG && signals) ? p->R * pl.ctpc : 0;
  const int words = workspace ? (int)((WS_HEADER_BYTES + pl.claim_bytes) / 4) : 0;   // header and piece claims
  if (std::max(words, n_sig) == 0) return FLUX_OK;
  hipLaunchKernelGGL(preset_kernel, dim3((std::max(words, n_sig) + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(stream), n_sig ? signals : (uint32_t*)nullptr, n_sig,
                     p->rank * pl.ctpc, (p->rank + 1) * pl.ctpc, static_cast<uint32_t*>(workspace), words);
  FLUX_HIP(hipGetLastError());
  return FLUX_OK;
}

int flux_tile_shape(int op, const flux_problem_t* p, int32_t* tile_m, int32_t* tile_n, int32_t* tile_k,
                    int32_t* split_k, int32_t* n_xcd) {
  Plan pl;
  int st = make_plan(op, p, &pl);
  if (st != FLUX_OK) return st;
  if (tile_m) *tile_m = pl.bm;
  if (tile_n) *tile_n = pl.bn;
  if (tile_k) *tile_k = pl.bk;
  if (split_k) *split_k = pl.split_k;
  if (n_xcd) *n_xcd = pl.n_xcd;
  return FLUX_OK;
}

int flux_split_plan(int op, const flux_problem_t* p, int32_t* full_tiles, int32_t* split_tiles, int32_t* split_k) {
  Plan pl;
  int st = make_plan(op, p, &pl);
  if (st != FLUX_OK) return st;
  if (full_tiles) *full_tiles = pl.full_tiles;
  if (split_tiles) *split_tiles = pl.split_tiles;
  if (split_k) *split_k = pl.split_k;
  return FLUX_OK;
}

int32_t flux_ag_deferred_tiles(const flux_problem_t* p) {
  Plan pl;
  if (p == nullptr || make_plan(FLUX_OP_AG, p, &pl) != FLUX_OK) return 0;
  return pl.defer_tiles;
}

int32_t flux_rs_resident_grid(const flux_problem_t* p, uint32_t* delay_ticks) {
  Plan pl;
  if (delay_ticks) *delay_ticks = 0;
  if (p == nullptr || make_plan(FLUX_OP_RS, p, &pl) != FLUX_OK || !pl.resident) return 0;
  if (delay_ticks) *delay_ticks = pl.resident_delay_ticks;
  return N_CU;
}

int flux_tile_coord(int op, const flux_problem_t* p, const int32_t* arrival_order, int32_t block,
                    int32_t* m_tile, int32_t* n_tile) {
  Plan pl;
  int st = make_plan(op, p, &pl);
  if (st != FLUX_OK) return st;
  if (!m_tile || !n_tile || block < 0 || block >= pl.tiles_m * pl.tiles_n) return FLUX_ERR_INVALID_ARG;
  int order[FLUX_MAX_RANKS];
  if (op == FLUX_OP_AG) {
    st = check_arrival(p, arrival_order, order);
    if (st != FLUX_OK) return st;
  }
  static thread_local TileMap tm;
  build_tile_map(op, p, pl, order, &tm);
  int mt, nt;
  tile_coord(tm, block, mt, nt);
  *m_tile = mt; *n_tile = nt;
  return FLUX_OK;
}

int flux_query_status(const void* workspace, int32_t* code, int32_t* detail) {
  if (workspace == nullptr || code == nullptr) return FLUX_ERR_INVALID_ARG;
  uint32_t h[2] = {0, 0};
  FLUX_HIP(hipMemcpy(h, static_cast<const unsigned char*>(workspace) + WS_STATUS_OFF, sizeof(h), hipMemcpyDeviceToHost));
  *code = (int32_t)h[0];
  if (detail) *detail = (int32_t)h[1];
  return FLUX_OK;
}

int flux_gemm_rs(const flux_problem_t* p, const void* A, const void* B, const void* const* peer_partials,
                 void* const* out_slices, void* workspace, size_t workspace_bytes, void* stream) {
  Plan pl;
  int st = make_plan(FLUX_OP_RS, p, &pl);
  if (st != FLUX_OK) return st;
  return gemm_rs_planned(p, pl, A, B, peer_partials, out_slices, workspace, workspace_bytes, stream);
}

int flux_gemm_rs_static(const flux_problem_t* p, const void* A, const void* B, const void* const* peer_partials,
                        void* const* out_slices, void* stream) {
  Plan pl;
  int st = make_plan(FLUX_OP_RS, p, &pl);
  if (st != FLUX_OK) return st;
  const size_t need = pl.split_k > 1 ? workspace_need(pl) : 0;
  if (need > (size_t)FLUX_STATIC_SCRATCH_BYTES) return FLUX_ERR_WORKSPACE;
  if (need == 0) return gemm_rs_planned(p, pl, A, B, peer_partials, out_slices, nullptr, 0, stream);
  void* scratch = nullptr;
  st = static_scratch(&scratch);
  if (st != FLUX_OK) return st;
  // The array keeps what the last call on this GPU left in it.  The arrival counters of the K-cut
  // tiles must start at zero (a call that was interrupted may have left some behind); the partials
  // are written before they are read.  A small kernel, not a memset: callers may be capturing.
  const int words = (int)(WS_HEADER_BYTES / 4);
  hipLaunchKernelGGL(preset_kernel, dim3((words + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                     (uint32_t*)nullptr, 0, 0, 0, static_cast<uint32_t*>(scratch), words);
  FLUX_HIP(hipGetLastError());
  return gemm_rs_planned(p, pl, A, B, peer_partials, out_slices, scratch, (size_t)FLUX_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"

namespace flux {

int gemm_rs_planned(const flux_problem_t* p, const Plan& pl, const void* A, const void* B, const void* const* peer_partials,
                    void* const* out_slices, void* workspace, size_t workspace_bytes, void* stream, uint32_t* tile_ready) {
  int st;
  const bool atomic = p->flags & FLUX_FLAG_RS_ATOMIC;
  if (atomic && ((p->flags & FLUX_FLAG_RS_WRITE_ONLY) || p->out_dtype != FLUX_F32)) return FLUX_ERR_UNSUPPORTED;
  const bool write_only = (p->flags & FLUX_FLAG_RS_WRITE_ONLY) || atomic;   // neither form reads peers
  if (!A || !B || (!peer_partials && !write_only) || !out_slices || !aligned16(A) || !aligned16(B)) return FLUX_ERR_INVALID_ARG;
  for (int r = 0; r < p->R; ++r) {
    if (!out_slices[r] || !aligned16(out_slices[r])) return FLUX_ERR_INVALID_ARG;
    if (!write_only && r != p->rank && (!peer_partials[r] || !aligned16(peer_partials[r]))) return FLUX_ERR_INVALID_ARG;
  }
  st = check_workspace(pl, FLUX_OP_RS, workspace, workspace_bytes);
  if (st != FLUX_OK) return st;
  flux_trace_record_t* trace;
  st = take_trace(pl, &trace);
  if (st != FLUX_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  GemmArgs a;
  fill_common(&a, p, pl, pl.split_k > 1 ? workspace : nullptr);
  a.trace = trace;
  a.tile_ready = tile_ready;
  a.A = static_cast<const __bf16*>(A);
  a.B = static_cast<const __bf16*>(B);
  // the kernel wants the R-1 peers packed, ascending rank
  a.write_only = atomic ? 2 : (write_only ? 1 : 0);
  for (int r = 0, j = 0; r < p->R; ++r) {
    a.outs[r] = out_slices[r];
    if (!write_only && r != p->rank) a.peers[j++] = peer_partials[r];
  }
  build_tile_map(FLUX_OP_RS, p, pl, nullptr, &a.tm);
  return launch_gemm(pl, EPI_RS, 0, a, s);
}

}  // namespace flux

extern "C" {

int32_t flux_rs_ready_count(const flux_problem_t* p) {
  Plan pl;
  if (make_plan(FLUX_OP_RS, p, &pl) != FLUX_OK) return 0;
  return pl.tiles_m * pl.tiles_n;
}

int flux_gemm_rs_notify(const flux_problem_t* p, const void* A, const void* B, void* const* out_slices,
                        uint32_t* tile_ready, void* workspace, size_t workspace_bytes, void* stream) {
  if (p == nullptr || tile_ready == nullptr) return FLUX_ERR_INVALID_ARG;
  if (p->flags & FLUX_FLAG_RS_ATOMIC) return FLUX_ERR_UNSUPPORTED;
  flux_problem_t q = *p;
  q.flags |= FLUX_FLAG_RS_WRITE_ONLY;
  Plan pl;
  int st = make_plan(FLUX_OP_RS, &q, &pl);
  if (st != FLUX_OK) return st;
  return gemm_rs_planned(&q, pl, A, B, nullptr, out_slices, workspace, workspace_bytes, stream, tile_ready);
}

int flux_rs_reduce_slice_ready(const flux_problem_t* p, const void* const* staged, void* out, uint32_t* tile_ready,
                               int32_t producers, void* workspace, size_t workspace_bytes, void* stream) {
  Plan pl;
  int st = make_plan(FLUX_OP_RS, p, &pl);
  if (st != FLUX_OK) return st;
  if (!staged || !out || !tile_ready || !aligned16(out) || producers < 1) return FLUX_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < WS_HEADER_BYTES || !aligned16(workspace)) return FLUX_ERR_WORKSPACE;
  ReadyReduceArgs r;
  std::memset(&r, 0, sizeof(r));
  for (int j = 0; j < p->R; ++j) {
    if (!staged[j] || !aligned16(staged[j])) return FLUX_ERR_INVALID_ARG;
    r.staged[j] = staged[j];
  }
  const int S = p->M / p->R;
  r.out = out;
  r.tile_ready = tile_ready;
  r.status = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace) + WS_STATUS_OFF);
  r.timeout_ticks = p->spin_timeout_ticks ? p->spin_timeout_ticks : DEFAULT_TIMEOUT_TICKS;
  r.S = S; r.N = p->N; r.R = p->R;
  r.ld = (int32_t)pitch_c(p);
  r.partial_f32 = p->partial_dtype == FLUX_F32;
  r.out_f32 = p->out_dtype == FLUX_F32;
  r.bm = pl.bm; r.bn = pl.bn; r.tiles_n = pl.tiles_n;
  r.row0 = p->rank * S;
  r.mt_lo = r.row0 / pl.bm;
  r.n_mt = (r.row0 + S - 1) / pl.bm - r.mt_lo + 1;
  r.producers = producers;
  // A small persistent grid: its workgroups wait on compute units that the producers' GEMM
  // workgroups (which take a whole unit each) then cannot use.
  const int grid = std::max(1, std::min(r.n_mt * pl.tiles_n, 32));
  hipLaunchKernelGGL(rs_ready_reduce_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), r);
  FLUX_HIP(hipGetLastError());
  return FLUX_OK;
}

int flux_ag_gemm(const flux_problem_t* p, const void* const* A_chunks, void* A_agg, const void* B, void* C,
                 uint32_t* signals, const int32_t* arrival_order, void* workspace, size_t workspace_bytes,
                 void* compute_stream, void* copy_stream) {
  Plan pl;
  int st = make_plan(FLUX_OP_AG, p, &pl);
  if (st != FLUX_OK) return st;
  if (!A_chunks || !A_agg || !B || !C || !signals || !aligned16(A_agg) || !aligned16(B) || !aligned16(C)) return FLUX_ERR_INVALID_ARG;
  if (compute_stream == copy_stream) return FLUX_ERR_INVALID_ARG;
  const size_t chunk_elems = (size_t)(p->M / p->R) * p->K;
  if ((chunk_elems / pl.ctpc) % 8 != 0) return FLUX_ERR_SHAPE;
  for (int r = 0; r < p->R; ++r)
    if (!A_chunks[r] || !aligned16(A_chunks[r])) return FLUX_ERR_INVALID_ARG;
  int order[FLUX_MAX_RANKS];
  st = check_arrival(p, arrival_order, order);
  if (st != FLUX_OK) return st;
  st = check_workspace(pl, FLUX_OP_AG, workspace, workspace_bytes);
  if (st != FLUX_OK) return st;
  flux_trace_record_t* trace;
  st = take_trace(pl, &trace);
  if (st != FLUX_OK) return st;
  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t xs = static_cast<hipStream_t>(copy_stream);

  GemmArgs a;
  fill_common(&a, p, pl, workspace);
  a.trace = trace;
  a.A = static_cast<const __bf16*>(A_agg);
  a.B = static_cast<const __bf16*>(B);
  a.C = C;
  a.signals = signals;
  a.n_signals = p->R * pl.ctpc;
  a.sig_local_lo = p->rank * pl.ctpc;
  a.sig_local_hi = (p->rank + 1) * pl.ctpc;
  // rows that do not start and end on cache line boundaries may share a line with a row of another
  // communication tile
  a.acquire_l2 = (reinterpret_cast<uintptr_t>(A_agg) % 128 != 0) || (((size_t)pitch_a(p) * 2) % 128 != 0);
  const uint32_t call_id = next_call_id();
  if (pl.copy_help && p->R > 1) {
    a.copy_pieces = pl.copy_pieces;
    a.copy_driver_wgs = pl.copy_self ? 0 : pl.copy_wgs;
    // A waiting workgroup holds a whole compute unit: unless the driver stands for a link of a given
    // rate, it moves pieces of what it waits for right away instead of spinning next to the driver.
    a.copy_eager = pl.copy_self || p->link_gbps == 0;
    a.copy_call_id = pl.copy_self ? 0u : call_id;   // without a copy kernel the id lives in the workspace
    a.copy_call_seq = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace) + WS_CALLSEQ_OFF);
    a.copy_tile_vec = (unsigned long long)chunk_elems / 8 / pl.ctpc;
    for (int r = 0; r < p->R; ++r) a.outs[r] = const_cast<void*>(A_chunks[r]);   // chunk sources by rank
    if (pl.copy_self) {
      a.copy_owner_wgs = pl.copy_owners;
      a.copy_n_tiles = (p->R - 1) * pl.ctpc;
      a.copy_defer_tiles = pl.defer_tiles;
      a.copy_defer_steps = pl.defer_steps;
      a.copy_pace_ticks = pl.pace_ticks;
      static_assert(FLUX_MAX_RANKS <= 16, "chunk indices are packed four bits each");
      for (int i = 0; i < p->R - 1; ++i) a.copy_order4 |= (unsigned long long)order[i] << (4 * i);
    }
  }
  if ((p->flags & FLUX_FLAG_COPY_MEMCPY) && p->R > 1) {
    // the grid moves nothing unless the library copies are starved of compute units: then, after
    // 100 us without a signal, a workgroup fetches its own rows
    for (int r = 0; r < p->R; ++r) a.outs[r] = const_cast<void*>(A_chunks[r]);   // chunk sources by rank
    a.self_serve_ticks = 10000u;
  }
  build_tile_map(FLUX_OP_AG, p, pl, order, &a.tm);

  const bool driver_form = !(pl.copy_self || p->R == 1);
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  if (driver_form) {
    // The forms with a driver beside the grid take a claim id from the host and fork onto a second
    // stream: recorded in a graph, every replay would find all pieces claimed already.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    FLUX_HIP(hipStreamIsCapturing(cs, &cap));
    if (cap != hipStreamCaptureStatusNone) return FLUX_ERR_UNSUPPORTED;
    st = get_events(&ev_fork, &ev_join);
    if (st != FLUX_OK) return st;
  }

  // local chunk (its signal is preset, so it must be in place before the kernel starts)
  const __bf16* local_dst = static_cast<const __bf16*>(A_agg) + (size_t)p->rank * (p->M / p->R) * pitch_a(p);
  if (A_chunks[p->rank] != static_cast<const void*>(local_dst)) {
    int self = p->rank;
    st = launch_copy(p, pl, A_chunks, A_agg, &self, 1, false, nullptr, nullptr, 0, cs);
    if (st != FLUX_OK) return st;
  }
  if (!driver_form) {
    // nothing runs beside the GEMM grid: no fork, no join
    return launch_gemm(pl, EPI_PLAIN, 1, a, cs);
  }
  // fork: the copy driver may start once everything queued so far on compute_stream is done
  FLUX_HIP(hipEventRecord(ev_fork, cs));
  FLUX_HIP(hipStreamWaitEvent(xs, ev_fork, 0));
  if (p->flags & FLUX_FLAG_COPY_MEMCPY) {
    const size_t tile_bytes = chunk_elems * 2 / pl.ctpc;
    for (int i = 0; i < p->R - 1; ++i) {
      const int c = order[i];
      for (int t = 0; t < pl.ctpc; ++t) {
        const unsigned char* src = static_cast<const unsigned char*>(A_chunks[c]) + (size_t)t * tile_bytes;
        const size_t rows = (size_t)(p->M / p->R) / pl.ctpc, row_bytes = (size_t)p->K * 2, pitch = (size_t)pitch_a(p) * 2;
        unsigned char* dst = static_cast<unsigned char*>(A_agg) + ((size_t)c * pl.ctpc + t) * rows * pitch;
        if (pitch == row_bytes) FLUX_HIP(hipMemcpyAsync(dst, src, tile_bytes, hipMemcpyDeviceToDevice, xs));
        else FLUX_HIP(hipMemcpy2DAsync(dst, pitch, src, row_bytes, row_bytes, rows, hipMemcpyDeviceToDevice, xs));
        FLUX_HIP(hipStreamWriteValue32(xs, signals + c * pl.ctpc + t, 1u, 0));
      }
    }
  } else {
    st = launch_copy(p, pl, A_chunks, A_agg, order, p->R - 1, true, signals, workspace, call_id, xs);
    if (st != FLUX_OK) return st;
  }
  st = launch_gemm(pl, EPI_PLAIN, 1, a, cs);
  if (st != FLUX_OK) return st;
  // join: compute_stream continues only after the copy driver has finished too (the signals
  // were already put back by the last workgroup past its wait)
  FLUX_HIP(hipEventRecord(ev_join, xs));
  FLUX_HIP(hipStreamWaitEvent(cs, ev_join, 0));
  if (p->flags & FLUX_FLAG_COPY_MEMCPY) {
    // a copy that the grid overtook (its workgroups fetched their rows themselves) writes its signal
    // after the grid's own reset: put the array back once more behind the join (Sec. 4.3: the
    // reset after the GEMM, with a stream and an event)
    hipLaunchKernelGGL(preset_kernel, dim3((a.n_signals + 255) / 256), dim3(256), 0, cs, signals, a.n_signals,
                       a.sig_local_lo, a.sig_local_hi, (uint32_t*)nullptr, 0);
    FLUX_HIP(hipGetLastError());
  }
  return FLUX_OK;
}

int flux_gemm_ref_unfused(int op, int phases, const flux_problem_t* p, const void* A, const void* const* A_chunks,
                          void* A_agg, const void* B, const void* const* peer_partials, void* const* out_slices,
                          void* C, void* workspace, size_t workspace_bytes, void* stream) {
  Plan pl;
  int st = make_plan(op, p, &pl);
  if (st != FLUX_OK) return st;
  if ((phases & (FLUX_PHASE_GEMM | FLUX_PHASE_COMM)) == 0 || (phases & ~(FLUX_PHASE_GEMM | FLUX_PHASE_COMM))) return FLUX_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool do_gemm = phases & FLUX_PHASE_GEMM, do_comm = phases & FLUX_PHASE_COMM;
  if (!C || !aligned16(C)) return FLUX_ERR_INVALID_ARG;
  if (do_gemm) {
    if (!B || !aligned16(B)) return FLUX_ERR_INVALID_ARG;
    if (pl.split_k > 1) {
      if (workspace == nullptr || workspace_bytes < workspace_need(pl)) return FLUX_ERR_WORKSPACE;
    }
  }
  flux_trace_record_t* trace = nullptr;
  if (do_gemm) {
    st = take_trace(pl, &trace);
    if (st != FLUX_OK) return st;
  }
  GemmArgs a;
  fill_common(&a, p, pl, pl.split_k > 1 ? workspace : nullptr);
  a.trace = trace;
  a.B = static_cast<const __bf16*>(B);
  a.C = C;
  // natural tile order for the baseline GEMM, die remap kept
  flux_problem_t q = *p;
  q.flags |= FLUX_FLAG_NO_SWIZZLE;
  Plan plq = pl;
  build_tile_map(op, &q, plq, nullptr, &a.tm);
  a.tm.n_xcd = pl.n_xcd;
  a.tm.band_h = 1;

  if (op == FLUX_OP_RS) {
    if (do_gemm) {
      if (!A || !aligned16(A)) return FLUX_ERR_INVALID_ARG;
      a.A = static_cast<const __bf16*>(A);
      st = launch_gemm(pl, EPI_PLAIN, 0, a, s);
      if (st != FLUX_OK) return st;
    }
    if (do_comm) {
      if (!peer_partials || !out_slices) return FLUX_ERR_INVALID_ARG;
      ReduceArgs r;
      std::memset(&r, 0, sizeof(r));
      for (int j = 0; j < p->R; ++j) {
        if (!out_slices[j] || !aligned16(out_slices[j])) return FLUX_ERR_INVALID_ARG;
        if (j != p->rank && (!peer_partials[j] || !aligned16(peer_partials[j]))) return FLUX_ERR_INVALID_ARG;
        r.peers[j] = peer_partials[j];
        r.outs[j] = out_slices[j];
      }
      r.C = C; r.M = p->M; r.N = p->N; r.R = p->R; r.rank = p->rank; r.S = p->M / p->R;
      r.partial_f32 = p->partial_dtype == FLUX_F32;
      r.out_f32 = p->out_dtype == FLUX_F32;
      r.c_f32 = r.out_f32;
      r.ld_c = (int32_t)pitch_c(p); r.ld_peer = p->N; r.ld_out = (int32_t)pitch_c(p);
      r.row0 = 0; r.rows = p->M;
      const long long nvec = (long long)p->M * p->N / 8;
      const int grid = (int)std::min<long long>((nvec + 255) / 256, 256 * 8);
      hipLaunchKernelGGL(rs_reduce_kernel, dim3(grid), dim3(256), 0, s, r);
      FLUX_HIP(hipGetLastError());
    }
    return FLUX_OK;
  }
  // AllGather: copy every chunk, then the GEMM
  if (!A_agg || !aligned16(A_agg)) return FLUX_ERR_INVALID_ARG;
  if (do_comm) {
    if (!A_chunks) return FLUX_ERR_INVALID_ARG;
    int order[FLUX_MAX_RANKS];
    int n = 0;
    const size_t chunk_elems = (size_t)(p->M / p->R) * p->K;
    if (chunk_elems % 8 != 0) return FLUX_ERR_SHAPE;
    for (int r = 0; r < p->R; ++r) {
      if (!A_chunks[r] || !aligned16(A_chunks[r])) return FLUX_ERR_INVALID_ARG;
      const void* dst = static_cast<const __bf16*>(A_agg) + (size_t)r * (p->M / p->R) * pitch_a(p);
      if (A_chunks[r] != dst) order[n++] = r;
    }
    st = launch_copy(p, pl, A_chunks, A_agg, order, n, false, nullptr, nullptr, 0, s);
    if (st != FLUX_OK) return st;
  }
  if (do_gemm) {
    a.A = static_cast<const __bf16*>(A_agg);
    st = launch_gemm(pl, EPI_PLAIN, 0, a, s);
    if (st != FLUX_OK) return st;
  }
  return FLUX_OK;
}

int flux_rs_reduce_slice(const flux_problem_t* p, const void* const* staged, void* out, void* stream) {
  int st = validate_problem(FLUX_OP_RS, p);
  if (st != FLUX_OK) return st;
  if (!staged || !out || !aligned16(out)) return FLUX_ERR_INVALID_ARG;
  ReduceArgs r;
  std::memset(&r, 0, sizeof(r));
  for (int j = 0; j < p->R; ++j) {
    if (!staged[j] || !aligned16(staged[j])) return FLUX_ERR_INVALID_ARG;
    r.peers[j] = staged[j];
  }
  // one slice of S rows: the first partial plays the part of C, the others are added in rank order
  const int S = p->M / p->R;
  r.C = staged[0];
  r.outs[0] = out;
  r.M = S; r.N = p->N; r.R = p->R; r.rank = 0; r.S = S;
  r.partial_f32 = p->partial_dtype == FLUX_F32;
  r.c_f32 = r.partial_f32;
  r.out_f32 = p->out_dtype == FLUX_F32;
  r.ld_c = r.ld_peer = r.ld_out = (int32_t)pitch_c(p);
  r.row0 = 0; r.rows = S;
  const long long nvec = (long long)S * p->N / 8;
  const int grid = (int)std::max<long long>(1, std::min<long long>((nvec + 255) / 256, 256 * 8));
  hipLaunchKernelGGL(rs_reduce_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), r);
  FLUX_HIP(hipGetLastError());
  return FLUX_OK;
}

static flux_problem_t chunk_problem(const flux_problem_t* p) {
  flux_problem_t q = *p;
  q.M = p->M / p->R; q.R = 1; q.rank = 0;
  q.flags = FLUX_FLAG_NO_SWIZZLE;
  return q;
}

size_t flux_chunked_workspace_bytes(int op, const flux_problem_t* p) {
  if (validate_problem(op, p) != FLUX_OK) return 0;
  flux_problem_t q = chunk_problem(p);
  Plan plq;
  if (make_plan(FLUX_OP_RS, &q, &plq) != FLUX_OK || plq.split_k <= 1) return 0;
  return workspace_need(plq);
}

int flux_gemm_ref_chunked(int op, const flux_problem_t* p, const void* A, const void* const* A_chunks, void* A_agg,
                          const void* B, const void* const* peer_partials, void* const* out_slices, void* C,
                          const int32_t* arrival_order, void* workspace, size_t workspace_bytes,
                          void* compute_stream, void* comm_stream) {
  int st = validate_problem(op, p);
  if (st != FLUX_OK) return st;
  if (!B || !C || !aligned16(B) || !aligned16(C)) return FLUX_ERR_INVALID_ARG;
  if (compute_stream == comm_stream) return FLUX_ERR_INVALID_ARG;
  hipStream_t cs = static_cast<hipStream_t>(compute_stream), xs = static_cast<hipStream_t>(comm_stream);
  const int R = p->R, S = p->M / p->R;
  const size_t out_size = p->out_dtype == FLUX_F32 ? 4 : 2;

  // one rank-less GEMM of S rows per chunk, planned like any other GEMM of that shape
  flux_problem_t q = chunk_problem(p);
  Plan plq;
  st = make_plan(FLUX_OP_RS, &q, &plq);
  if (st != FLUX_OK) return st;
  if (plq.split_k > 1 && (workspace == nullptr || workspace_bytes < workspace_need(plq) || !aligned16(workspace)))
    return FLUX_ERR_WORKSPACE;
  GemmArgs g;
  fill_common(&g, &q, plq, plq.split_k > 1 ? workspace : nullptr);
  g.B = static_cast<const __bf16*>(B);
  build_tile_map(FLUX_OP_RS, &q, plq, nullptr, &g.tm);
  g.tm.n_xcd = plq.n_xcd;
  g.tm.band_h = 1;

  hipEvent_t* ev;
  st = get_chunk_events(&ev);
  if (st != FLUX_OK) return st;
  hipEvent_t ev_fork, ev_join;
  st = get_events(&ev_fork, &ev_join);
  if (st != FLUX_OK) return st;

  if (op == FLUX_OP_RS) {
    if (!A || !aligned16(A) || !peer_partials || !out_slices) return FLUX_ERR_INVALID_ARG;
    ReduceArgs r;
    std::memset(&r, 0, sizeof(r));
    for (int j = 0; j < R; ++j) {
      if (!out_slices[j] || !aligned16(out_slices[j])) return FLUX_ERR_INVALID_ARG;
      if (j != p->rank && (!peer_partials[j] || !aligned16(peer_partials[j]))) return FLUX_ERR_INVALID_ARG;
      r.peers[j] = peer_partials[j];
      r.outs[j] = out_slices[j];
    }
    r.C = C; r.M = p->M; r.N = p->N; r.R = R; r.rank = p->rank; r.S = S;
    r.partial_f32 = p->partial_dtype == FLUX_F32;
    r.out_f32 = p->out_dtype == FLUX_F32;
    r.c_f32 = r.out_f32;
    r.ld_c = (int32_t)pitch_c(p); r.ld_peer = p->N; r.ld_out = (int32_t)pitch_c(p);
    const long long nvec = (long long)S * p->N / 8;
    const int grid = (int)std::max<long long>(1, std::min<long long>((nvec + 255) / 256, 256 * 8));
    // slices in the order of the fused kernel: the ring after the local rank, the own slice last
    for (int d = 1; d <= R; ++d) {
      const int slice = (p->rank + d) % R;
      g.A = static_cast<const __bf16*>(A) + (size_t)slice * S * pitch_a(p);
      g.C = static_cast<unsigned char*>(C) + (size_t)slice * S * pitch_c(p) * out_size;
      st = launch_gemm(plq, EPI_PLAIN, 0, g, cs);
      if (st != FLUX_OK) return st;
      FLUX_HIP(hipEventRecord(ev[slice], cs));
      FLUX_HIP(hipStreamWaitEvent(xs, ev[slice], 0));
      r.row0 = slice * S; r.rows = S;
      hipLaunchKernelGGL(rs_reduce_kernel, dim3(grid), dim3(256), 0, xs, r);
      FLUX_HIP(hipGetLastError());
    }
    FLUX_HIP(hipEventRecord(ev_join, xs));
    FLUX_HIP(hipStreamWaitEvent(cs, ev_join, 0));
    return FLUX_OK;
  }

  // AllGather: chunk copies on comm_stream in arrival order, each chunk's GEMM once its copy is done
  if (!A_chunks || !A_agg || !aligned16(A_agg)) return FLUX_ERR_INVALID_ARG;
  const size_t chunk_elems = (size_t)S * p->K;
  if (chunk_elems % 8 != 0) return FLUX_ERR_SHAPE;
  for (int r = 0; r < R; ++r)
    if (!A_chunks[r] || !aligned16(A_chunks[r])) return FLUX_ERR_INVALID_ARG;
  int order[FLUX_MAX_RANKS];
  st = check_arrival(p, arrival_order, order);
  if (st != FLUX_OK) return st;
  Plan plc;                                   // only its copy parameters are used
  st = make_plan(FLUX_OP_AG, p, &plc);
  if (st != FLUX_OK) return st;
  const __bf16* agg = static_cast<const __bf16*>(A_agg);
  if (A_chunks[p->rank] != static_cast<const void*>(agg + (size_t)p->rank * S * pitch_a(p))) {
    int self = p->rank;
    st = launch_copy(p, plc, A_chunks, A_agg, &self, 1, false, nullptr, nullptr, 0, cs);
    if (st != FLUX_OK) return st;
  }
  FLUX_HIP(hipEventRecord(ev_fork, cs));
  FLUX_HIP(hipStreamWaitEvent(xs, ev_fork, 0));
  for (int i = 0; i < R - 1; ++i) {
    const int c = order[i];
    st = launch_copy(p, plc, A_chunks, A_agg, &c, 1, false, nullptr, nullptr, 0, xs);
    if (st != FLUX_OK) return st;
    FLUX_HIP(hipEventRecord(ev[c], xs));
  }
  for (int i = -1; i < R - 1; ++i) {
    const int c = i < 0 ? p->rank : order[i];
    if (i >= 0) FLUX_HIP(hipStreamWaitEvent(cs, ev[c], 0));
    g.A = agg + (size_t)c * S * pitch_a(p);
    g.C = static_cast<unsigned char*>(C) + (size_t)c * S * pitch_c(p) * out_size;
    st = launch_gemm(plq, EPI_PLAIN, 0, g, cs);
    if (st != FLUX_OK) return st;
  }
  return FLUX_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------
// tuner (Sec. 4.4; communication tile size: Sec. 4.3)
// ------------------------------------------------------------------------------------------
namespace {

struct Candidate { int32_t tile_config, ctpc, split_k; uint32_t flags = 0; };   // flags: added to the caller's

// Every tile configuration that accepts the shape; for AllGather each with the communication tile
// halved from the chunk down to the GEMM tile height (Sec. 4.3), at most 8 tiles per chunk.
std::vector<Candidate> tune_candidates(int op, const flux_problem_t* p) {
  std::vector<Candidate> out;
  const int S = p->M / p->R;
  for (int cfg = 1; cfg <= NUM_CFGS; ++cfg) {
    flux_problem_t q = *p;
    q.tile_config = cfg;
    q.split_k = 0;
    q.comm_tiles_per_chunk = 0;
    Plan pl;
    if (make_plan(op, &q, &pl) != FLUX_OK) continue;
    out.push_back({cfg, 1, 0});
    // the forms of prologue and epilogue the plan would pick by rule are knobs too (Sec. 4.4): all chunks
    // moved before the first main loop instead of carried inside it; one workgroup per tile instead of
    // a resident grid
    if (op == FLUX_OP_AG && pl.defer_tiles > 0 && pl.pace_ticks == 0) out.push_back({cfg, 1, 0, FLUX_FLAG_AG_COPY_UPFRONT});
    if (op == FLUX_OP_RS && pl.resident) out.push_back({cfg, 1, 0, FLUX_FLAG_NO_RESIDENT_GRID});
    // few rows: how K is cut decides how well the grid fills the chip and what the hand-over costs;
    // half and twice the library's number of parts are candidates too
    if (p->M <= 256 && pl.full_tiles == 0) {
      const int kt = (p->K + pl.bk - 1) / pl.bk;
      for (int sk : {pl.split_k / 2, pl.split_k * 2}) {
        if (sk < 1 || sk == pl.split_k || sk > 64 || sk > kt / 4) continue;
        flux_problem_t r = q;
        r.split_k = sk;
        Plan plr;
        if (make_plan(op, &r, &plr) == FLUX_OK && plr.split_k == sk) out.push_back({cfg, 1, sk});
      }
    }
    if (op != FLUX_OP_AG) continue;
    for (int t = 2; t <= 8; t *= 2) {
      if (S % t != 0 || S / t < pl.bm || p->R * t > MAX_COMM_TILES) break;
      out.push_back({cfg, t, 0});
    }
  }
  return out;
}

struct TuneBuffers {
  const void* A; const void* const* A_chunks; void* A_agg; const void* B;
  const void* const* peers; void* const* outs; void* C; uint32_t* signals; const int32_t* arrival;
  void* ws; size_t ws_bytes; void* cs; void* xs;
};

int tune_call(int op, const flux_problem_t* q, const TuneBuffers& b) {
  if (op == FLUX_OP_RS) return flux_gemm_rs(q, b.A, b.B, b.peers, b.outs, b.ws, b.ws_bytes, b.cs);
  return flux_ag_gemm(q, b.A_chunks, b.A_agg, b.B, b.C, b.signals, b.arrival, b.ws, b.ws_bytes, b.cs, b.xs);
}

// median time per call in ms of `reps` samples, each a batch of back-to-back calls long enough to time
int tune_time(int op, const flux_problem_t* q, const TuneBuffers& b, int reps, hipEvent_t e0, hipEvent_t e1, float* ms_out) {
  hipStream_t cs = static_cast<hipStream_t>(b.cs);
  int st = flux_init_buffers(op, q, b.ws, b.ws_bytes, op == FLUX_OP_AG ? b.signals : nullptr, b.cs);
  if (st != FLUX_OK) return st;
  int batch = 1;
  std::vector<float> samples;
  for (int r = -2; r < reps; ++r) {          // two warm-up samples; the first also sizes the batch
    FLUX_HIP(hipEventRecord(e0, cs));
    for (int i = 0; i < batch; ++i) {
      st = tune_call(op, q, b);
      if (st != FLUX_OK) return st;
    }
    FLUX_HIP(hipEventRecord(e1, cs));
    FLUX_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    FLUX_HIP(hipEventElapsedTime(&ms, e0, e1));
    if (b.ws != nullptr && op == FLUX_OP_AG) {
      int32_t code = 0, detail = 0;
      st = flux_query_status(b.ws, &code, &detail);
      if (st != FLUX_OK) return st;
      if (code != FLUX_OK) return code;
    }
    if (r == -2) batch = std::max(2, std::min(32, (int)(2.0f / std::max(ms, 1e-3f))));   // samples of about 2 ms, calls back to back
    else if (r >= 0) samples.push_back(ms / (float)batch);
  }
  std::sort(samples.begin(), samples.end());
  *ms_out = samples[samples.size() / 2];
  return FLUX_OK;
}

int tune(int op, const flux_problem_t* p, const TuneBuffers& b, int reps, flux_problem_t* tuned, float* ms_best,
         float* ms_default) {
  if (p == nullptr || tuned == nullptr) return FLUX_ERR_INVALID_ARG;
  if (reps <= 0) reps = 5;
  reps = std::min(reps, 100);
  Plan pl;
  int st = make_plan(op, p, &pl);
  if (st != FLUX_OK) return st;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  FLUX_HIP(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FLUX_ERR_HIP; }
  flux_problem_t base = *p;        // what the library picks by itself
  base.tile_config = 0; base.split_k = 0; base.comm_tiles_per_chunk = 0;
  float t_default = 0.f;
  st = tune_time(op, &base, b, reps, e0, e1, &t_default);
  flux_problem_t best = base;
  float t_best = t_default;
  if (st == FLUX_OK) {
    for (const Candidate& c : tune_candidates(op, p)) {
      flux_problem_t q = base;
      q.tile_config = c.tile_config;
      q.comm_tiles_per_chunk = c.ctpc;
      q.split_k = c.split_k;
      q.flags |= c.flags;
      if (flux_workspace_bytes(op, &q) > b.ws_bytes) continue;     // the caller's workspace does not hold this one
      float t = 0.f;
      const int sc = tune_time(op, &q, b, reps, e0, e1, &t);
      if (sc == FLUX_ERR_HIP) { st = sc; break; }
      if (sc != FLUX_OK) continue;                                  // e.g. timed out: not a candidate
      if (t < t_best * 0.98f) { t_best = t; best = q; }             // the library's own pick wins ties
    }
  }
  if (st == FLUX_OK) {
    // the library's pick once more, now that clocks and caches are where the candidates found them
    float t_again = 0.f;
    st = tune_time(op, &base, b, reps, e0, e1, &t_again);
    if (st == FLUX_OK && t_again < t_default) {
      t_default = t_again;
      if (best.tile_config == 0 && best.comm_tiles_per_chunk == 0 && best.split_k == 0 && best.flags == base.flags) t_best = t_again;
      else if (t_best >= t_default * 0.98f) { best = base; t_best = t_default; }
    }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != FLUX_OK) return st;
  // leave the buffers ready for calls with the tuned problem
  st = flux_init_buffers(op, &best, b.ws, b.ws_bytes, op == FLUX_OP_AG ? b.signals : nullptr, b.cs);
  if (st != FLUX_OK) return st;
  FLUX_HIP(hipStreamSynchronize(static_cast<hipStream_t>(b.cs)));
  *tuned = best;
  if (ms_best) *ms_best = t_best;
  if (ms_default) *ms_default = t_default;
  return FLUX_OK;
}

}  // namespace

extern "C" {

size_t flux_autotune_workspace_bytes(int op, const flux_problem_t* p) {
  if (p == nullptr) return 0;
  flux_problem_t base = *p;
  base.tile_config = 0; base.split_k = 0; base.comm_tiles_per_chunk = 0;
  size_t need = flux_workspace_bytes(op, &base);
  for (const Candidate& c : tune_candidates(op, p)) {
    flux_problem_t q = base;
    q.tile_config = c.tile_config;
    q.comm_tiles_per_chunk = c.ctpc;
    q.split_k = c.split_k;
    need = std::max(need, flux_workspace_bytes(op, &q));
  }
  return need;
}

int flux_autotune_signal_count(const flux_problem_t* p) {
  if (p == nullptr || p->R < 1) return 0;
  int t_max = 1;
  for (const Candidate& c : tune_candidates(FLUX_OP_AG, p)) t_max = std::max(t_max, (int)c.ctpc);
  return p->R * t_max;
}

int flux_autotune_rs(const flux_problem_t* p, const void* A, const void* B, const void* const* peer_partials,
                     void* const* out_slices, void* workspace, size_t workspace_bytes, void* stream, int32_t reps,
                     flux_problem_t* tuned, float* ms_best, float* ms_default) {
  TuneBuffers b{};
  b.A = A; b.B = B; b.peers = peer_partials; b.outs = out_slices; b.ws = workspace; b.ws_bytes = workspace_bytes; b.cs = stream;
  return tune(FLUX_OP_RS, p, b, reps, tuned, ms_best, ms_default);
}

int flux_autotune_ag(const flux_problem_t* p, const void* const* A_chunks, void* A_agg, const void* B, void* C,
                     uint32_t* signals, int32_t signal_count, const int32_t* arrival_order, void* workspace,
                     size_t workspace_bytes, void* compute_stream, void* copy_stream, int32_t reps,
                     flux_problem_t* tuned, float* ms_best, float* ms_default) {
  if (p == nullptr || signals == nullptr || signal_count < flux_autotune_signal_count(p)) return FLUX_ERR_INVALID_ARG;
  TuneBuffers b{};
  b.A_chunks = A_chunks; b.A_agg = A_agg; b.B = B; b.C = C; b.signals = signals; b.arrival = arrival_order;
  b.ws = workspace; b.ws_bytes = workspace_bytes; b.cs = compute_stream; b.xs = copy_stream;
  return tune(FLUX_OP_AG, p, b, reps, tuned, ms_best, ms_default);
}

}  // extern "C"
