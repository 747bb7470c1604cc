// Device-side building blocks of the fused tensor-parallel GEMM kernels (gfx950 / CDNA4).
//
// One templated kernel serves the three entry points; what differs is the prologue
// (AllGather-GEMM waits on signals, paper Alg. 2) and the epilogue (GEMM-ReduceScatter adds
// the peer partial tiles and writes each row into its owner's slice, paper Alg. 1).
//
// Mapping to the hardware:
//   * bf16 inputs, v_mfma_f32_32x32x16_bf16, fp32 accumulators kept in registers;
//   * A tile [BM][BK] and B tile [BK][BN] staged in LDS with XOR-swizzled 16-byte slots;
//     A fragments are read with ds_read_b128, B fragments (B is [K,N] row-major, so a lane
//     needs 8 consecutive k of one column) with the transposing ds_read_b64_tr_b16;
//   * 128-bit global loads into registers for tile t+1 while tile t is multiplied;
//   * the accumulators go through LDS once in the epilogue so that every lane owns 8
//     consecutive columns of a row: peer partials are read and outputs written 16 B (bf16)
//     or 32 B (fp32) per lane, 128..512 B contiguous per row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "flux.h"

namespace flux {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// ---- workspace layout (bytes) -------------------------------------------------------------
constexpr size_t WS_STATUS_OFF = 0;        // uint32 code, uint32 detail
constexpr size_t WS_DONE_OFF = 16;         // uint32: workgroups that are past their signal wait
constexpr size_t WS_STARTED_OFF = 32;      // uint32: copy-driver workgroups that have started
constexpr size_t WS_CALLSEQ_OFF = 48;      // uint32: calls without a copy kernel that have completed on this workspace
constexpr size_t WS_COUNTER_OFF = 256;     // uint32 per communication tile (copy kernel arrivals)
constexpr int MAX_COMM_TILES = 1024;
constexpr size_t WS_TILECNT_OFF = WS_COUNTER_OFF + 4 * MAX_COMM_TILES;   // split-K arrival counters
constexpr int MAX_SPLITK_TILES = 4096;
// Workgroups past their signal wait are counted in two levels: workgroup b adds to leaf b mod
// DONE_LEAVES, whoever completes a leaf adds to the root (WS_DONE_OFF).  Hundreds of additions to one
// address queue up behind each other (tens of nanoseconds each), and every workgroup waits for its
// own to come back.  The leaves lie in different memory channels.
constexpr int DONE_LEAVES = 32;
constexpr size_t DONE_LEAF_STRIDE = 256;
constexpr size_t WS_DONELEAF_OFF = WS_TILECNT_OFF + 4 * MAX_SPLITK_TILES;
constexpr size_t WS_HEADER_BYTES = WS_DONELEAF_OFF + DONE_LEAVES * DONE_LEAF_STRIDE;
// After the header: AllGather piece claims (uint32 per communication tile and piece), then the
// split-K partials.
constexpr int MAX_COPY_PIECES = 256;       // pieces per communication tile = copy-driver workgroups

// ---- TileCoord (paper Sec. 4.1) -----------------------------------------------------------
// The host builds `m_order`: the order in which m-tiles are scheduled (slice by slice after
// the local rank for ReduceScatter, chunk by chunk in arrival order for AllGather).  Ascending
// workgroup ids walk that order in bands of `band_h` m-tiles times all n-tiles, m fastest.
// Workgroups are dealt round-robin to the accelerator dies, so with n_xcd > 1 the in-band index
// is regrouped to give every die a contiguous run of the band (shared panels stay in its L2).
// With at most 16 m-tiles the order also sits in `order4`, four bits per position: a kernel then
// has its tile after the first fetch of its arguments, not after a second, dependent one into the
// table (about a microsecond at the start of every workgroup).
struct TileMap {
  int32_t tiles_m, tiles_n, band_h, n_xcd;
  int32_t packed, pad_;
  uint64_t order4;
  uint16_t m_order[FLUX_MAX_M_TILES];
};

__host__ __device__ inline void tile_coord(const TileMap& tm, int block, int& mt, int& nt) {
  const int band_sz = tm.band_h * tm.tiles_n;
  const int band = block / band_sz;
  int q = block - band * band_sz;
  if (tm.n_xcd > 1 && band_sz % tm.n_xcd == 0) q = (q % tm.n_xcd) * (band_sz / tm.n_xcd) + q / tm.n_xcd;
  const int i = band * tm.band_h + q % tm.band_h;
  nt = q / tm.band_h;
  mt = tm.packed ? (int)((tm.order4 >> (4 * i)) & 15) : (int)tm.m_order[i];
}

enum : int { EPI_PLAIN = 0, EPI_RS = 1 };

// Kernel arguments.  A workgroup's first fetches from the argument block miss the scalar cache one
// 64-byte line after the other, a quarter of a microsecond each, before its first load can be
// issued: the scalars sit together at the front, grouped by who needs them (every kernel; the signal
// wait; the transfer; split-K and the reduce-scatter epilogue), and the arrays come last.
struct GemmArgs {
  // ---- every kernel ----
  const __bf16* A;           // [M,K]
  const __bf16* B;           // [K,N]
  void* C;                   // [M,N] of out dtype (plain epilogue)
  int32_t M, N, K;
  int32_t R, rank, S;        // S = M / R
  int32_t lda, ldb, ldc;     // row pitches in elements: A (the gathered matrix); B; C and the out slices (peer partials are packed)
  int32_t b_is_nk;           // B is [N,K] (the kernels built for that layout are launched)
  // K split: the first `full_tiles` tiles (in TileCoord order) are computed by one workgroup
  // each; every one of the remaining `split_tiles` tiles by `split_k` workgroups that each take
  // `k_per_split` of K.  A uniform split has full_tiles = 0; splitting only the tiles of the last,
  // partly filled round of the grid keeps all CUs busy to the end.
  int32_t full_tiles, split_tiles;
  int32_t split_k, k_per_split;   // k_per_split is a multiple of BK
  // ---- all-gather prologue: the signal wait ----
  uint32_t* signals;
  uint32_t* done_counter;
  uint32_t* status;
  unsigned long long timeout_ticks;
  int32_t rows_per_signal;
  int32_t n_signals, sig_local_lo, sig_local_hi;   // local communication tiles: [lo, hi)
  // the transfer: pieces of communication tiles are claimed and moved by this grid's workgroups
  // and/or a copy kernel (outs[] then holds the chunk sources, A is the gathered matrix);
  // copy_pieces = 0: the grid moves nothing and only waits (hipMemcpyAsync driver, or R = 1)
  int32_t copy_pieces;       // pieces per communication tile
  // No driver at all (copy_owner_wgs > 0): piece g (counted over the remote communication tiles in
  // transfer order, tile j lying in the chunk at position j / ctpc of copy_order4) belongs to
  // workgroup g % copy_owner_wgs of this grid, which moves it before it looks at its own signals.
  int32_t copy_owner_wgs;
  int32_t copy_eager;        // waiting workgroups take pieces even while the whole driver is running
  int32_t acquire_l2;        // the gathered rows may share cache lines across communication tiles: full acquire after the wait
  // The driver is a copy engine or library copy that takes no pieces (copy_pieces = 0): a workgroup
  // that has waited this long (100 MHz ticks; 0: never) fetches the rows of its own tile itself.
  uint32_t self_serve_ticks;
  // ---- the transfer ----
  uint32_t* copy_claims;     // [n_signals][copy_pieces], a piece is taken when it holds copy_call_id
  uint32_t* copy_counters;   // [n_signals] pieces finished
  uint32_t* copy_call_seq;
  uint32_t* started_counter;
  unsigned long long copy_order4;   // chunk of position i in bits [4i, 4i+4)
  unsigned long long copy_tile_vec;   // 16-byte vectors per communication tile
  uint32_t copy_call_id;     // 0: take the id from copy_call_seq (calls without a copy kernel)
  int32_t copy_driver_wgs;   // workgroups of the copy kernel launched beside this grid (0: none)
  int32_t copy_n_tiles;
  // The last copy_defer_tiles remote communication tiles of the transfer order are not moved before
  // the signal wait: the workgroups of the first round carry them inside their main loops (piece w
  // of each such tile by workgroup w, copy_defer_steps 16-byte vectors per thread and tile).
  int32_t copy_defer_tiles;
  int32_t copy_defer_steps;
  // ... and with copy_pace_ticks != 0 they stand for a link: the i-th tile of the transfer order is
  // counted in no earlier than (i + 1) * copy_pace_ticks (100 MHz ticks) after the kernel started
  unsigned long long copy_pace_ticks;
  // ---- split-K hand-over, reduce-scatter epilogue ----
  int32_t write_only;        // 1: reduce-scatter epilogue without the reduction (Write branch of Alg. 1);
                             // 2: no peers are read, the tile is added to the slice with atomic additions
  float* sk_partials;             // [split_k][split_tiles][BM*BN] fp32
  uint32_t* sk_counters;          // [tiles]
  int32_t partial_f32, out_f32;
  flux_trace_record_t* trace;     // tile trace, one record per workgroup; null: none
  uint32_t* tile_ready;           // reduce-scatter, Write branch: per output tile, producers that have written it; null: not kept
  int32_t persist_blocks;         // > 0: a grid of resident workgroups, workgroup b takes the blocks b, b + grid, ... below this
  uint32_t persist_delay_ticks;   // ... and every second group of eight starts this late (100 MHz ticks)
  // ---- arrays ----
  void* outs[FLUX_MAX_RANKS];
  const void* peers[FLUX_MAX_RANKS];   // the R-1 peer partials packed in ascending rank order
  TileMap tm;
};

// The rank-indexed pointers (output slices, or chunk sources) go to LDS for dynamic indexing.  The
// second half of the array lies in another line of the argument block and is only touched when
// there are that many ranks.  Made visible to the other threads by the next workgroup barrier.
__device__ __forceinline__ void fill_lds_outs(const GemmArgs& a, void** lds_outs, int tid) {
  static_assert(FLUX_MAX_RANKS == 16, "two halves of eight");
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (tid == j) lds_outs[j] = a.outs[j];
  if (a.R > 8) {
#pragma unroll
    for (int j = 8; j < 16; ++j)
      if (tid == j) lds_outs[j] = a.outs[j];
  }
}

// workgroup id -> (tile in TileCoord order, K split index, is this tile split)
__device__ __forceinline__ void map_block(const GemmArgs& a, int b, int& tile, int& split, bool& is_split) {
  if (b < a.full_tiles) {
    tile = b; split = 0; is_split = false;
  } else {
    const int r = b - a.full_tiles;
    tile = a.full_tiles + r % a.split_tiles;
    split = r / a.split_tiles;
    is_split = a.split_k > 1;
  }
}

// ---- tile trace -------------------------------------------------------------------------------
// With a trace buffer every workgroup leaves one record: which tile and K part it computed, on which
// die and compute unit, and the 100 MHz wall clock at four points (kernel entry, past the signal
// wait, main loop done, epilogue stores acknowledged).  Thread 0 writes; without a buffer the cost
// is one scalar test per point.
enum : int { TRACE_START = 0, TRACE_READY = 1, TRACE_MAIN_END = 2, TRACE_END = 3 };

__device__ __forceinline__ void trace_begin(const GemmArgs& a, int tile, int mt, int nt, int split, bool is_split, int vb = -1) {
  if (a.trace == nullptr || threadIdx.x != 0) return;
  const uint32_t b = vb < 0 ? blockIdx.x : (uint32_t)vb;
  flux_trace_record_t* r = a.trace + b;
  r->block = b;
  r->m_tile = (uint32_t)mt;
  r->n_tile = (uint32_t)nt;
  r->k_part = (uint32_t)split | (is_split ? 0x10000u : 0u);
  r->die = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) ;       // XCC_ID, bits [3:0]
  r->hw_id = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));      // HW_ID, all 32 bits
  r->tile = (uint32_t)tile;
  r->reserved = 0;
  const uint64_t t = wall_clock64();
  r->t_start = t; r->t_ready = t; r->t_main_end = t; r->t_end = t;
}

__device__ __forceinline__ void trace_stamp(const GemmArgs& a, int point, int vb = -1) {
  if (a.trace == nullptr) return;
  if (point == TRACE_END) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's stores are acknowledged
  if (threadIdx.x != 0) return;
  flux_trace_record_t* r = a.trace + (vb < 0 ? blockIdx.x : (uint32_t)vb);
  const uint64_t t = wall_clock64();
  if (point == TRACE_READY) r->t_ready = t;
  if (point <= TRACE_MAIN_END) r->t_main_end = t;
  r->t_end = t;
}

// ---- LDS swizzles ---------------------------------------------------------------------------
// A tile: rows of BK bf16 = BK/8 slots of 16 B; slot s of row r is stored at slot s ^ fA(r).
// With 128-byte rows, 8 (or 16) consecutive rows read the same logical slot in one
// ds_read_b128 pass; fA spreads them over all banks for both a 128 B and a 256 B wide LDS.
template <int SLOTS>
__device__ __forceinline__ int swz_a(int row) {
  return ((row & 7) ^ ((row >> 3) & 1)) & (SLOTS - 1);
}
// B tile: rows of BN bf16 (one k each); the transposing read touches 4 consecutive k rows at
// the same columns, so rows k..k+3 are pushed to different 64-byte (and 32-byte) bank groups.
template <int SLOTS>
__device__ __forceinline__ int swz_b(int k) {
  const int kk = k & 3;
  return ((kk << 2) ^ (kk << 1)) & (SLOTS - 1);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 h = __builtin_convertvector(v, bf16x2);   // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, h);
}

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Streaming (non-temporal) 16-byte accesses for data touched exactly once: peer partials and
// outputs must not push the A/B panels, which are re-read many times, out of the L2.
__device__ __forceinline__ uint4 ld_stream16(const void* p) {
  const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void st_stream16(void* p, const uint4& v) {
  const u32x4 d = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(d, static_cast<u32x4*>(p));
}

// 16-byte store at device scope: written through this die's L2, so that a reader on another
// accelerator die needs no write-back of the whole L2 to see it.
__device__ __forceinline__ void store_through(uint4* p, const u32x4& d) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(d) : "memory");
}
// Output vectors: streamed, or written through when a consumer may read the tile as soon as its ready
// counter moves (`through`, uniform).
__device__ __forceinline__ void st_out16(void* p, const uint4& v, bool through) {
  if (through) store_through(static_cast<uint4*>(p), u32x4{v.x, v.y, v.z, v.w});
  else st_stream16(p, v);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// B_NK: B is given as [N,K] (row n holds the K values of output column n, the layout of a linear
// layer's weight).  Its tile then sits in LDS like A's (rows of BK values, the same slot swizzle) and a
// fragment is one 16-byte read per lane, as for A, instead of two transposing reads.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int NSTAGE_, int OCC_, bool B_NK_ = false>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NSTAGE = NSTAGE_, OCC = OCC_;
  static constexpr bool B_NK = B_NK_;
  static constexpr int NT = WAVES_M * WAVES_N * 64;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static constexpr int A_SLOTS = BK / 8, B_SLOTS = BN / 8;
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BK * BN * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int A_VEC = BM * BK / 8 / NT, B_VEC = BK * BN / 8 / NT;
  static constexpr int EP_STRIDE = WTN + 8;                       // floats; 4 rows apart = 128 B off
  static constexpr int EP_BYTES = WAVES_M * WAVES_N * 32 * EP_STRIDE * 4;
  static constexpr int ESTAGE = NSTAGE >= 2 ? 2 : 1;              // stages of the register-staged kernel
  static constexpr int MAIN_BYTES = ESTAGE * STAGE_BYTES > EP_BYTES ? ESTAGE * STAGE_BYTES : EP_BYTES;
  static constexpr int MISC_OFF = MAIN_BYTES;              // 16 B: one int shared by the workgroup
  static constexpr int PTRS_OFF = MAIN_BYTES + 16;         // FLUX_MAX_RANKS output slice pointers
  static constexpr int LDS_BYTES = PTRS_OFF + 8 * FLUX_MAX_RANKS;
  static_assert(BM % (WAVES_M * 32) == 0 && BN % (WAVES_N * 32) == 0 && BK % 16 == 0, "tile shape");
  static_assert((BM * BK / 8) % NT == 0 && (BK * BN / 8) % NT == 0, "loader shape");
  static_assert(B_SLOTS >= 8, "BN >= 64");
};

template <class C, bool EDGE>
struct Loader {
  // per-thread global pointers of the 16-byte vectors this thread stages, k offset 0
  const __bf16* pa[C::A_VEC];
  const __bf16* pb[C::B_VEC];
  int lds_a[C::A_VEC], lds_b[C::B_VEC];
  int ka[C::A_VEC];            // column (k) offset of each A vector inside the tile
  int kb[C::B_VEC];            // row (k) offset of each B vector inside the tile
  bool nb_ok[C::B_VEC];

  __device__ __forceinline__ void init(const GemmArgs& a, int m0, int n0, int tid) {
#pragma unroll
    for (int p = 0; p < C::A_VEC; ++p) {
      const int v = tid + C::NT * p;
      const int row = v / C::A_SLOTS, slot = v % C::A_SLOTS;
      int gr = m0 + row;
      if (EDGE) gr = gr < a.M ? gr : a.M - 1;
      pa[p] = a.A + (size_t)gr * a.lda + slot * 8;
      ka[p] = slot * 8;
      lds_a[p] = row * (C::BK * 2) + ((slot ^ swz_a<C::A_SLOTS>(row)) << 4);
    }
#pragma unroll
    for (int p = 0; p < C::B_VEC; ++p) {
      const int v = tid + C::NT * p;
      if constexpr (C::B_NK) {
        const int n = v / C::A_SLOTS, slot = v % C::A_SLOTS;
        int gn = n0 + n;
        nb_ok[p] = !EDGE || gn < a.N;
        if (EDGE && gn >= a.N) gn = 0;
        pb[p] = a.B + (size_t)gn * a.ldb + slot * 8;
        kb[p] = slot * 8;
        lds_b[p] = C::A_BYTES + n * (C::BK * 2) + ((slot ^ swz_a<C::A_SLOTS>(n)) << 4);
      } else {
        const int k = v / C::B_SLOTS, s = v % C::B_SLOTS;
        int gn = n0 + s * 8;
        nb_ok[p] = !EDGE || gn < a.N;
        if (EDGE && gn >= a.N) gn = 0;
        pb[p] = a.B + (size_t)k * a.ldb + gn;
        kb[p] = k;
        lds_b[p] = C::A_BYTES + k * (C::BN * 2) + ((s ^ swz_b<C::B_SLOTS>(k)) << 4);
      }
    }
  }

  __device__ __forceinline__ void load(const GemmArgs& a, int k0, int k_end, uint4 (&ra)[C::A_VEC], uint4 (&rb)[C::B_VEC]) const {
#pragma unroll
    for (int p = 0; p < C::A_VEC; ++p) {
      if (!EDGE || k0 + ka[p] < k_end) ra[p] = *reinterpret_cast<const uint4*>(pa[p] + k0);
      else ra[p] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int p = 0; p < C::B_VEC; ++p) {
      if (!EDGE || (nb_ok[p] && k0 + kb[p] < k_end))
        rb[p] = *reinterpret_cast<const uint4*>(pb[p] + (C::B_NK ? (size_t)k0 : (size_t)k0 * a.ldb));
      else rb[p] = make_uint4(0, 0, 0, 0);
    }
  }

  __device__ __forceinline__ void store(unsigned char* stage, const uint4 (&ra)[C::A_VEC], const uint4 (&rb)[C::B_VEC]) const {
#pragma unroll
    for (int p = 0; p < C::A_VEC; ++p) *reinterpret_cast<uint4*>(stage + lds_a[p]) = ra[p];
#pragma unroll
    for (int p = 0; p < C::B_VEC; ++p) *reinterpret_cast<uint4*>(stage + lds_b[p]) = rb[p];
  }
};

// One BK-deep slab of MFMAs out of the LDS stage.
template <class C>
__device__ __forceinline__ void mma_stage(const unsigned char* stage, int wm, int wn, int lane,
                                          f32x16 (&acc)[C::MI][C::NI]) {
  const int g = lane >> 4, i = lane & 15;
#pragma unroll
  for (int ks = 0; ks < C::BK / 16; ++ks) {
    bf16x8 af[C::MI], bfr[C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
      const int row = wm * C::WTM + mi * 32 + (lane & 31);
      const int q = ks * 2 + (lane >> 5);
      af[mi] = *reinterpret_cast<const bf16x8*>(stage + row * (C::BK * 2) + ((q ^ swz_a<C::A_SLOTS>(row)) << 4));
    }
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      if constexpr (C::B_NK) {
        const int row = wn * C::WTN + ni * 32 + (lane & 31);
        const int q = ks * 2 + (lane >> 5);
        bfr[ni] = *reinterpret_cast<const bf16x8*>(stage + C::A_BYTES + row * (C::BK * 2) + ((q ^ swz_a<C::A_SLOTS>(row)) << 4));
      } else {
        const int k = ks * 16 + 8 * (g >> 1) + (i >> 2);
        const int n = wn * C::WTN + ni * 32 + 16 * (g & 1) + 4 * (i & 3);
        const int off = C::A_BYTES + k * (C::BN * 2) + ((((n >> 3) ^ swz_b<C::B_SLOTS>(k))) << 4) + ((n >> 2) & 1) * 8;
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(stage + off));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(stage + off + 4 * C::BN * 2));
        s16x8 w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bfr[ni] = __builtin_bit_cast(bf16x8, w);
      }
    }
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
  }
}

// Store 8 consecutive output columns of one row into the owner's slice (GetOutput of Alg. 1) or
// into C, converting once.
template <int EPI>
__device__ __forceinline__ void store_row8(const GemmArgs& a, void* const* lds_outs, int gm, int gn, const float (&v)[8]) {
  void* base;
  size_t o;
  const bool through = EPI == EPI_RS && a.tile_ready != nullptr;
  if (EPI == EPI_RS) {
    const int r = gm / a.S;
    base = lds_outs[r];
    o = (size_t)(gm - r * a.S) * a.ldc + gn;
  } else {
    base = a.C;
    o = (size_t)gm * a.ldc + gn;
  }
  if (a.out_f32) {
    float* q = static_cast<float*>(base) + o;
    st_out16(q, make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])), through);
    st_out16(q + 4, make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])), through);
  } else {
    uint4 w;
    w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
    w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
    st_out16(static_cast<__bf16*>(base) + o, w, through);
  }
}

// The peer partials of one tile as buffer resources based at the tile's origin (Reduce of Alg. 1
// reads them).  `a.peers` holds the R-1 peers in ascending rank order; a resource past that has no
// records, so its loads return zeros and every lane runs the same straight-line code: seven loads
// per 8-column piece, no branch and no pointer fetch between them.
struct PeerBufs {
  __amdgpu_buffer_rsrc_t r[FLUX_MAX_RANKS - 1];
};

__device__ __forceinline__ void make_peer_bufs(const GemmArgs& a, int m0, int n0, PeerBufs& pb) {
  const size_t tile_off = ((size_t)m0 * a.N + n0) * (a.partial_f32 ? 4 : 2);
#pragma unroll
  for (int j = 0; j < FLUX_MAX_RANKS - 1; ++j) {
    // (the address is the same in every lane; saying so keeps the resource in scalar registers)
    const uint64_t addr = reinterpret_cast<uint64_t>(a.peers[j]) + tile_off;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)addr), hi = __builtin_amdgcn_readfirstlane((uint32_t)(addr >> 32));
    unsigned char* base = reinterpret_cast<unsigned char*>(((uint64_t)hi << 32) | lo);
    pb.r[j] = __builtin_amdgcn_make_buffer_rsrc(base, 0, j < a.R - 1 ? 0x7fffffff : 0, 0x00027000);
  }
}

// One 32-row block of a wave's tile, already transposed into `ep`: every lane takes 8 consecutive
// columns of a row per pass.  With the reduce-scatter epilogue the peer loads of BATCH passes are
// issued together before any of them is used (PF32: fp32 partials, two 16-byte loads per peer);
// the peers are added in ascending rank order.
template <class C, int EPI, bool EDGE, bool PF32, int BATCH, int NP>
__device__ __forceinline__ void epilogue_block(const GemmArgs& a, void* const* lds_outs, const float* ep, const PeerBufs& pb,
                                               int row_base, int col_base, int m0, int n0, int lane) {
  constexpr int CH = C::WTN / 8;          // 8-column pieces per row of the wave tile
  constexpr int RPP = 64 / CH;            // rows per pass
  constexpr int NIT = 32 / RPP;
  constexpr int B = BATCH < NIT ? BATCH : NIT;
  constexpr int LPP = PF32 ? 2 : 1;
  constexpr int NT_HINT = 2;              // cache policy: streamed once, do not keep
  static_assert(NIT % B == 0, "batch must divide the passes");
  const int cc = lane % CH, rl = lane / CH;
#pragma unroll
  for (int it0 = 0; it0 < NIT; it0 += B) {
    u32x4 w[B][NP > 0 ? NP : 1][LPP];
    bool ok[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int row = row_base + (it0 + b) * RPP + rl, col = col_base + cc * 8;
      ok[b] = !EDGE || (m0 + row < a.M && n0 + col < a.N);
      if (EPI == EPI_RS) {
        // a lane outside the matrix gets an offset past the records: zeros, no memory access
        // (tile-relative: row < BM <= 256 and N < 2^21, so the byte offset stays below 2^31)
        const int voff = ok[b] ? (int)(((uint32_t)row * (uint32_t)a.N + (uint32_t)col) * (PF32 ? 4u : 2u)) : (int)0x80000000;
#pragma unroll
        for (int j = 0; j < NP; ++j)
#pragma unroll
          for (int l = 0; l < LPP; ++l) w[b][j][l] = __builtin_amdgcn_raw_buffer_load_b128(pb.r[j], voff + 16 * l, 0, NT_HINT);
      }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int r = (it0 + b) * RPP + rl;
      const float4 x = *reinterpret_cast<const float4*>(ep + r * C::EP_STRIDE + cc * 8);
      const float4 y = *reinterpret_cast<const float4*>(ep + r * C::EP_STRIDE + cc * 8 + 4);
      float v[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
      if (EPI == EPI_RS) {
#pragma unroll
        for (int j = 0; j < NP; ++j) {
          if (PF32) {
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[e] += __uint_as_float(w[b][j][0][e]); v[4 + e] += __uint_as_float(w[b][j][LPP - 1][e]); }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[2 * e] += bf16_lo(w[b][j][0][e]); v[2 * e + 1] += bf16_hi(w[b][j][0][e]); }
          }
        }
      }
      if (ok[b]) store_row8<EPI>(a, lds_outs, m0 + row_base + r, n0 + col_base + cc * 8, v);
    }
    // one batch of peer loads in flight at a time: left alone, the scheduler hoists the loads of
    // later batches up here too and has to spill accumulators to make room for them
    if (EPI == EPI_RS) __builtin_amdgcn_sched_barrier(0);
  }
}

// The whole epilogue of one wave: its accumulators pass through LDS 32 rows at a time.
template <class C, int EPI, bool EDGE, bool PF32, int BATCH, int NP>
__device__ __forceinline__ void epilogue_all(const GemmArgs& a, void* const* lds_outs, float* ep, f32x16 (&acc)[C::MI][C::NI],
                                             int m0, int n0, int lane, int wm, int wn) {
  PeerBufs pb;
  if (EPI == EPI_RS) make_peer_bufs(a, m0, n0, pb);
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi) {
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        ep[r * C::EP_STRIDE + ni * 32 + (lane & 31)] = acc[mi][ni][e];
      }
    __builtin_amdgcn_wave_barrier();
    epilogue_block<C, EPI, EDGE, PF32, BATCH, NP>(a, lds_outs, ep, pb, wm * C::WTM + mi * 32, wn * C::WTN, m0, n0, lane);
    __builtin_amdgcn_wave_barrier();
  }
}

// ---- AllGather copy pieces --------------------------------------------------------------------
// A communication tile is moved in `pieces` pieces; piece w is what workgroup w of a grid of
// `pieces` workgroups of 256 threads touches in a grid-stride loop over 16-byte vectors.  The copy
// driver's workgroup w normally moves piece w of every tile; a GEMM workgroup that would otherwise
// only wait may take pieces nobody has claimed yet.  Either way the piece is claimed first (a
// compare-and-swap of the call's id into the piece's claim word), moved, and counted in; whoever
// counts in last sets the tile's signal (SetSignal of Alg. 3).

// DEPTH vectors per thread in flight (32 made the plain chunk copy slower: 60 against 24 us for 58.7 MB);
// the last batch is predicated, not walked one vector (one memory round trip) at a time.
//
// The sources are packed; the gathered matrix may have a row pitch.  Vector i of a communication
// tile then goes to row i / kv, place i % kv, counted from the tile's first row.
struct AggPitch {
  uint32_t kv, pitch_v;      // 16-byte vectors per row; from one row to the next
  __device__ __forceinline__ bool packed() const { return kv == pitch_v; }
};
__device__ __forceinline__ AggPitch agg_pitch(const GemmArgs& a) { return AggPitch{(uint32_t)a.K / 8u, (uint32_t)a.lda / 8u}; }
// first vector of communication tile f in the gathered matrix
__device__ __forceinline__ uint4* agg_tile(const GemmArgs& a, int f) {
  return reinterpret_cast<uint4*>(const_cast<__bf16*>(a.A)) + (unsigned long long)f * a.rows_per_signal * ((unsigned long long)a.lda / 8);
}
template <bool PITCHED>
__device__ __forceinline__ unsigned long long agg_index(const AggPitch& g, unsigned long long i) {
  if (!PITCHED) return i;
  const uint32_t j = (uint32_t)i;          // a tile has fewer than 2^28 vectors
  return (unsigned long long)(j / g.kv) * g.pitch_v + j % g.kv;
}

template <int DEPTH, bool PITCHED>
__device__ __forceinline__ void copy_piece_as(const uint4* __restrict__ src, uint4* __restrict__ dst, unsigned long long tile_vec,
                                              int piece, int pieces, int tid, const AggPitch& g) {
  const unsigned long long stride = (unsigned long long)pieces * 256;
  for (unsigned long long i = (unsigned long long)piece * 256 + tid; i < tile_vec; i += DEPTH * stride) {
    u32x4 v[DEPTH];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u)
      if (i + u * stride < tile_vec) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + i + u * stride));
#pragma unroll
    for (int u = 0; u < DEPTH; ++u)
      if (i + u * stride < tile_vec) store_through(dst + agg_index<PITCHED>(g, i + u * stride), v[u]);
  }
}
template <int DEPTH = 16>
__device__ __forceinline__ void copy_piece(const uint4* __restrict__ src, uint4* __restrict__ dst, unsigned long long tile_vec,
                                           int piece, int pieces, int tid, const AggPitch& g) {
  if (g.packed()) copy_piece_as<DEPTH, false>(src, dst, tile_vec, piece, pieces, tid, g);       // (uniform)
  else copy_piece_as<DEPTH, true>(src, dst, tile_vec, piece, pieces, tid, g);
}

// A piece of at most COPY_DEPTH * 256 vectors in two halves: the loads, and, once the piece is known
// to be the caller's, the stores.  The loads touch only the source, so they can be on their way
// while the claim is.
constexpr int COPY_DEPTH = 16;
__device__ __forceinline__ void load_piece(const uint4* __restrict__ src, unsigned long long tile_vec, int piece, int pieces,
                                           int tid, u32x4 (&v)[COPY_DEPTH]) {
  const unsigned long long stride = (unsigned long long)pieces * 256;
  const unsigned long long i = (unsigned long long)piece * 256 + tid;
#pragma unroll
  for (int u = 0; u < COPY_DEPTH; ++u) {
    v[u] = u32x4{0, 0, 0, 0};
    if (i + u * stride < tile_vec) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + i + u * stride));
  }
}
template <bool PITCHED>
__device__ __forceinline__ void store_piece_as(uint4* __restrict__ dst, unsigned long long tile_vec, int piece, int pieces,
                                               int tid, const u32x4 (&v)[COPY_DEPTH], const AggPitch& g) {
  const unsigned long long stride = (unsigned long long)pieces * 256;
  const unsigned long long i = (unsigned long long)piece * 256 + tid;
#pragma unroll
  for (int u = 0; u < COPY_DEPTH; ++u)
    if (i + u * stride < tile_vec) store_through(dst + agg_index<PITCHED>(g, i + u * stride), v[u]);
}
__device__ __forceinline__ void store_piece(uint4* __restrict__ dst, unsigned long long tile_vec, int piece, int pieces,
                                            int tid, const u32x4 (&v)[COPY_DEPTH], const AggPitch& g) {
  if (g.packed()) store_piece_as<false>(dst, tile_vec, piece, pieces, tid, v, g);               // (uniform)
  else store_piece_as<true>(dst, tile_vec, piece, pieces, tid, v, g);
}

// true if the caller now owns the piece.  One exchange, one round trip: whoever swaps the call's id
// in first sees something else come back; anyone later swaps the id for itself.
__device__ __forceinline__ bool claim_piece(uint32_t* claim, uint32_t call_id) {
  return __hip_atomic_exchange(claim, call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != call_id;
}

// After the stores of `n` pieces of one tile: wait until they are acknowledged, count the pieces
// in, set the signal if they were the tile's last.  All threads of the workgroup call this.
__device__ __forceinline__ void finish_pieces(uint32_t* counter, uint32_t* signal, int pieces, int n) {
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's write-through stores are acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    if (n == pieces) {
      // the whole tile was this workgroup's (a small transfer: one piece per tile): nobody else counts, no round trip
      __hip_atomic_store(signal, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    } else {
      const uint32_t prev = __hip_atomic_fetch_add(counter, (uint32_t)n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (prev + (uint32_t)n == (uint32_t)pieces) {
        __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        __hip_atomic_store(signal, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
  }
  // Callers loop: without a barrier here, this one-thread block and the one-thread block that
  // opens the caller's next iteration (a claim, a counter fetch) are adjacent across the back
  // edge, and the compiler has been seen to merge them into one divergent region that the other
  // lanes of the first wave skip on their way to the next iteration's barrier, which they then
  // reach without thread 0 (and read what it has not written yet).
  __syncthreads();
}

// The copy driver's workgroups count themselves in when they start: word 0 of `started` only ever
// grows.  Word 1 is what word 0 read before the current call's driver was launched; the last GEMM
// workgroup past its wait advances it by the driver's size for the next call (by then every driver
// workgroup of this call has been or will be counted, and the next call starts after the driver
// has finished).  Nothing is ever reset, so a workgroup that starts late cannot spoil a count.
__device__ __forceinline__ bool driver_fully_started(const uint32_t* started, int workgroups) {
  if (workgroups == 0) return false;
  const uint32_t total = __hip_atomic_load(started, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint32_t base = __hip_atomic_load(started + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return total - base >= (uint32_t)workgroups;
}

// The id that marks a piece as taken in this call.  With a copy kernel beside the grid the host
// hands out a fresh one per call.  Without, it is the number of such calls that have completed on
// this workspace (the last workgroup past its wait counts the call in, when every workgroup has
// read the old value: a workgroup only reads it before it is past its own wait), so a call
// recorded in a graph gets a new id on every replay.
__device__ __forceinline__ uint32_t transfer_call_id(const GemmArgs& a) {
  if (a.copy_call_id != 0u) return a.copy_call_id;
  return 0x80000000u | __hip_atomic_load(a.copy_call_seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// No driver: the first copy_owner_wgs workgroups of the grid share the transfer out among
// themselves by index, each moving its pieces in transfer order before it looks at its own
// signals, whatever its own tile needs.  A piece still goes through the claim table (one word per
// piece, so nobody contends), which lets any waiting workgroup take over the piece of an owner
// that has not been given a compute unit yet.  The first wave claims up to 64 pieces in one round
// trip and, when they have been moved, counts them in in another.  `lds` is 4 ints shared by the
// workgroup; `lds_srcs` holds the chunk sources by rank (written before, not yet synchronised).
__device__ __forceinline__ void transfer_own_pieces(const GemmArgs& a, int* lds, void* const* lds_srcs) {
  if ((int)blockIdx.x >= a.copy_owner_wgs) return;
  const int tid = threadIdx.x;
  const int ctpc = a.n_signals / a.R;
  const int total = (a.copy_n_tiles - a.copy_defer_tiles) * a.copy_pieces;
  const int G = a.copy_owner_wgs;
  if (total <= G && a.copy_tile_vec <= (unsigned long long)a.copy_pieces * 256 * COPY_DEPTH) {
    // A small transfer (decode): at most one piece per owner, moved in one pass.  Then the whole
    // call waits for a chain of memory round trips, so they overlap where they can: the piece is
    // loaded while the call's id and then the claim are on their way.
    const int g = (int)blockIdx.x;
    if (g >= total) return;
    __syncthreads();                       // lds_srcs
    const uint32_t call_id = transfer_call_id(a);
    const int j = g / a.copy_pieces, piece = g - j * a.copy_pieces;
    const int chunk = (int)((a.copy_order4 >> (4 * (j / ctpc))) & 15), t = j % ctpc;
    const int f = chunk * ctpc + t;
    const uint4* src = static_cast<const uint4*>(lds_srcs[chunk]) + (unsigned long long)t * a.copy_tile_vec;
    uint4* dst = agg_tile(a, f);
    u32x4 v[COPY_DEPTH];
    load_piece(src, a.copy_tile_vec, piece, a.copy_pieces, tid, v);
    if (tid == 0) lds[2] = claim_piece(a.copy_claims + (size_t)f * a.copy_pieces + piece, call_id) ? 1 : 0;
    __syncthreads();
    if (lds[2]) {
      store_piece(dst, a.copy_tile_vec, piece, a.copy_pieces, tid, v, agg_pitch(a));
      finish_pieces(a.copy_counters + f, a.signals + f, a.copy_pieces, 1);
    }
    return;
  }
  const uint32_t call_id = transfer_call_id(a);
  for (int base = (int)blockIdx.x; base < total; base += 64 * G) {
    if (tid < 64) {
      const int g = base + tid * G;
      bool mine = false;
      if (g < total) {
        const int j = g / a.copy_pieces;
        const int f = (int)((a.copy_order4 >> (4 * (j / ctpc))) & 15) * ctpc + j % ctpc;
        mine = claim_piece(a.copy_claims + (size_t)f * a.copy_pieces + (g - j * a.copy_pieces), call_id);
      }
      const unsigned long long won = __ballot(mine);
      if (tid == 0) { lds[1] = (int)(uint32_t)won; lds[2] = (int)(uint32_t)(won >> 32); }
    }
    __syncthreads();
    const unsigned long long won = (unsigned long long)(uint32_t)lds[1] | ((unsigned long long)(uint32_t)lds[2] << 32);
    for (unsigned long long rest = won; rest != 0; rest &= rest - 1) {
      const int g = base + __builtin_ctzll(rest) * G;
      const int j = g / a.copy_pieces, piece = g - j * a.copy_pieces;
      const int chunk = (int)((a.copy_order4 >> (4 * (j / ctpc))) & 15), t = j % ctpc;
      const int f = chunk * ctpc + t;
      const uint4* src = static_cast<const uint4*>(lds_srcs[chunk]) + (unsigned long long)t * a.copy_tile_vec;
      copy_piece(src, agg_tile(a, f), a.copy_tile_vec, piece, a.copy_pieces, tid, agg_pitch(a));
    }
    // count the pieces in, all at once: lane l of the first wave for the piece it claimed
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's write-through stores are acknowledged
    __syncthreads();
    if (tid < 64 && ((won >> tid) & 1)) {
      const int g = base + tid * G;
      const int j = g / a.copy_pieces;
      const int f = (int)((a.copy_order4 >> (4 * (j / ctpc))) & 15) * ctpc + j % ctpc;
      const uint32_t prev = __hip_atomic_fetch_add(a.copy_counters + f, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (prev + 1u == (uint32_t)a.copy_pieces) {
        __hip_atomic_store(a.copy_counters + f, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        __hip_atomic_store(a.signals + f, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
    __syncthreads();
  }
}

// The transfer carried by the GEMM's own waves (Sec. 3.2: the tiles whose data has arrived compute
// while the rest is still on its way).  A workgroup of the first round owns piece `blockIdx.x` of
// every deferred communication tile and moves it in 16-byte vectors per thread, tile after tile in
// transfer order: inside its main loop two vectors per K slab (the loads at the end of a slab, the
// stores of what was loaded two slabs earlier at the start of one, so that neither is ever waited
// for), and in batches while it still waits for its own signals.  All addressing goes through
// buffer resources whose size is the tile's (or zero for a workgroup with nothing to move, a tile
// taken over by somebody else, or when all tiles are done), so a lane past the end, and everything
// such a workgroup issues, is dropped by the range check: the loops have one shape for every
// workgroup and no branch around a memory access.
// With a pace (the transfer stands for a link of a given rate) the data still moves as fast as the
// loops take it, but a tile is counted in, and so its signal set, no earlier than the link would
// have delivered it: tile number i of the transfer order (i + 1) * pace_ticks after the workgroup
// started (the workgroups of a first round start within a microsecond of each other).
struct SideCopy {
  __amdgpu_buffer_rsrc_t rs, rd;     // source chunk / its place in the gathered matrix, for the tile being loaded / stored
  uint32_t first, ld_off, st_off;    // this lane's first vector of a piece, next to load, next to store (byte offsets in the tile)
  uint32_t stride;                   // bytes between a lane's vectors
  int n_tiles, n_steps, pos0;        // deferred tiles; vectors per thread and tile; transfer position of the first of them
  int ld_t, ld_s, st_t, st_s;        // cursors: tile and step
  int fin_t;                         // tiles counted in so far
  uint32_t mine;                     // bit t: this workgroup claimed its piece of deferred tile t
  unsigned long long t0, pace;       // start clock; 100 MHz ticks per tile (0: unpaced)
  int* slot;                         // one int of LDS: whatever depends on the clock is decided by thread 0 and read from here

  // deferred tile t -> its signal index (= communication tile index in the gathered matrix) and chunk
  __device__ __forceinline__ void locate(const GemmArgs& a, int t, int& f, int& chunk, int& sub) const {
    const int ctpc = a.n_signals / a.R;
    const int pos = pos0 + t;
    chunk = (int)((a.copy_order4 >> (4 * (pos / ctpc))) & 15);
    sub = pos % ctpc;
    f = chunk * ctpc + sub;
  }
  __device__ __forceinline__ unsigned records(const GemmArgs& a, int t) const {
    return (t < n_tiles && ((mine >> t) & 1u)) ? (unsigned)(a.copy_tile_vec * 16ull) : 0u;
  }
  __device__ __forceinline__ void set_src(const GemmArgs& a, void* const* lds_srcs, int t) {
    int f = 0, chunk = 0, sub = 0;
    if (t < n_tiles) locate(a, t, f, chunk, sub);
    const uint64_t addr = reinterpret_cast<uint64_t>(lds_srcs[chunk]) + (unsigned long long)sub * a.copy_tile_vec * 16ull;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)addr), hi = __builtin_amdgcn_readfirstlane((uint32_t)(addr >> 32));
    rs = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0, (int)records(a, t), 0x00027000);
  }
  __device__ __forceinline__ void set_dst(const GemmArgs& a, int t) {
    int f = 0, chunk = 0, sub = 0;
    if (t < n_tiles) locate(a, t, f, chunk, sub);
    unsigned char* base = reinterpret_cast<unsigned char*>(const_cast<__bf16*>(a.A)) + (unsigned long long)f * a.copy_tile_vec * 16ull;
    rd = __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)records(a, t), 0x00027000);
  }

  // Claims this workgroup's pieces (one exchange per deferred tile, all in one round trip) and sets
  // the cursors up.  `lds` is one int shared by the workgroup, kept for this object.  All threads call this.
  __device__ __forceinline__ void begin(const GemmArgs& a, int* lds, void* const* lds_srcs) {
    const int tid = threadIdx.x;
    slot = lds;
    t0 = wall_clock64();
    pace = a.copy_pace_ticks;
    n_tiles = 0; mine = 0u; n_steps = a.copy_defer_steps;
    pos0 = a.copy_n_tiles - a.copy_defer_tiles;
    if (a.copy_defer_tiles > 0 && (int)blockIdx.x < a.copy_pieces && (int)blockIdx.x < a.copy_owner_wgs) n_tiles = a.copy_defer_tiles;
    if (n_tiles > 0) {           // (uniform)
      if (tid < 64) {
        bool won = false;
        if (tid < n_tiles) {
          int f, chunk, sub;
          locate(a, tid, f, chunk, sub);
          won = claim_piece(a.copy_claims + (size_t)f * a.copy_pieces + blockIdx.x, transfer_call_id(a));
        }
        const unsigned long long w = __ballot(won);
        if (tid == 0) *lds = (int)(uint32_t)w;
      }
      __syncthreads();
      mine = (uint32_t)__builtin_amdgcn_readfirstlane(*lds);
      __syncthreads();
    }
    first = ((uint32_t)blockIdx.x * 256u + (uint32_t)tid) * 16u;
    stride = (uint32_t)a.copy_pieces * 256u * 16u;
    ld_off = st_off = first;
    ld_t = ld_s = st_t = st_s = 0;
    fin_t = 0;
    if (mine == 0u) fin_t = n_tiles = 0;
    set_src(a, lds_srcs, 0);
    set_dst(a, 0);
  }
  __device__ __forceinline__ bool pending() const { return fin_t < n_tiles; }         // something left to move or to count in
  __device__ __forceinline__ bool all_stored() const { return st_t >= n_tiles; }
  // Is there a tile whose stores are all issued and which may be counted in now?  Reads the clock:
  // different waves may get different answers, so only thread 0's counts (see maybe_finish).
  __device__ __forceinline__ bool due() const {
    if (fin_t >= st_t) return false;
    if (pace == 0ull) return st_t >= n_tiles;        // unpaced: everything is counted in together, at the end
    return wall_clock64() - t0 >= (unsigned long long)(pos0 + fin_t + 1) * pace;
  }
  __device__ __forceinline__ bool may_be_due() const { return fin_t < st_t && (pace != 0ull || st_t >= n_tiles); }   // (uniform)

  __device__ __forceinline__ u32x4 load(const GemmArgs& a, void* const* lds_srcs) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)ld_off, 0, 2);      // streamed: not kept in the caches
    ld_off += stride;
    if (++ld_s == n_steps) { ld_s = 0; ld_off = first; set_src(a, lds_srcs, ++ld_t); }
    return v;
  }
  __device__ __forceinline__ void store(const GemmArgs& a, const u32x4& v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, rd, (int)st_off, 0, 16);                 // device scope: written through the die's L2
    st_off += stride;
    if (++st_s == n_steps) { st_s = 0; st_off = first; set_dst(a, ++st_t); }
  }
  // Counts in the tiles that are due (see due()).  A tile whose last piece this was gets its signal
  // (SetSignal of Alg. 3).  All threads call this.
  __device__ __forceinline__ void finish(const GemmArgs& a) {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's write-through stores are acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
      int upto = fin_t;
      const int stored = st_t < n_tiles ? st_t : n_tiles;
      if (pace == 0ull) {
        upto = stored;
      } else {
        const unsigned long long now = wall_clock64() - t0;
        while (upto < stored && now >= (unsigned long long)(pos0 + upto + 1) * pace) ++upto;
      }
      for (int t = fin_t; t < upto; ++t) {
        if (!((mine >> t) & 1u)) continue;
        int f, chunk, sub;
        locate(a, t, f, chunk, sub);
        const uint32_t prev = __hip_atomic_fetch_add(a.copy_counters + f, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev + 1u == (uint32_t)a.copy_pieces) {
          __hip_atomic_store(a.copy_counters + f, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
          __hip_atomic_store(a.signals + f, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
      }
      *slot = upto;
    }
    __syncthreads();
    fin_t = __builtin_amdgcn_readfirstlane(*slot);
    __syncthreads();                        // the slot is free again
  }
  // finish() if thread 0 finds a tile due.  All threads call this.
  __device__ __forceinline__ void maybe_finish(const GemmArgs& a) {
    if (!may_be_due()) return;
    __syncthreads();
    if (threadIdx.x == 0) *slot = due() ? 1 : 0;
    __syncthreads();
    const int go = __builtin_amdgcn_readfirstlane(*slot);
    __syncthreads();
    if (go) finish(a);
  }
  // While the workgroup has nothing else to do (it waits for its own signals, or its main loop is
  // over): a batch of vectors, loads first.  All threads call this.
  __device__ __forceinline__ void pump(const GemmArgs& a, void* const* lds_srcs) {
    constexpr int BATCH = 8;
    u32x4 v[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) v[u] = load(a, lds_srcs);
#pragma unroll
    for (int u = 0; u < BATCH; ++u) store(a, v[u]);
  }
  // Everything that is left, now: the rest of the vectors, then the tiles as they become due.
  // All threads call this.
  __device__ __forceinline__ void drain(const GemmArgs& a, void* const* lds_srcs) {
    while (ld_t < n_tiles) pump(a, lds_srcs);
    while (pending()) {
      maybe_finish(a);
      if (pending()) __builtin_amdgcn_s_sleep(16);
    }
  }
};

// Are the signals covering rows [m0, m1) all set?  One poll by the first wave, the answer handed to
// everybody through `slot` (one int of LDS).  All threads call this.
__device__ __forceinline__ bool signals_all_set(const GemmArgs& a, int m0, int m1, int* slot) {
  const int f0 = m0 / a.rows_per_signal, f1 = (m1 - 1) / a.rows_per_signal;
  const int nf = f1 - f0 + 1;
  if (threadIdx.x < 64) {
    bool any = false;
    for (int base = 0; base < nf; base += 64) {
      const bool unset = base + (int)threadIdx.x < nf &&
                         __hip_atomic_load(a.signals + f0 + base + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == 0u;
      any = any || __ballot(unset) != 0ull;
    }
    if (threadIdx.x == 0) *slot = any ? 0 : 1;
  }
  __syncthreads();
  const int all = __builtin_amdgcn_readfirstlane(*slot);
  __syncthreads();
  return all != 0;
}

// WaitSignal (Alg. 2).  The first wave polls the signals covering rows [m0, m1) with coherent
// loads, one lane per signal; when all are set, the workgroup barrier hands that to the other waves.
// A workgroup that finds a signal missing
// and unclaimed pieces among the tiles it waits for claims and moves such pieces itself (at once;
// beside a paced driver only while part of that driver has not been given a compute unit), picking
// them by a hash that depends on its index so that the workgroups of a grid spread over the pieces
// instead of racing for the same one: without that, a mover that never gets a compute unit (the
// GEMM grid may have taken them all, and its waiting workgroups do not leave) would stall the grid
// for good.  Bounded: past `timeout_ticks` the tile is given up and the status block says so.  A
// workgroup never looks at the signals again after this, so the last workgroup of the grid to get
// here puts the signal array back into its preset state for the next call (the reset "after the
// GEMM" of Sec. 4.3, without a separate launch).
// `lds` is 4 ints shared by the workgroup; `lds_srcs` holds the chunk sources by rank.
__device__ __forceinline__ bool wait_signals(const GemmArgs& a, int m0, int m1, int* lds, void* const* lds_srcs) {
  const int tid = threadIdx.x;
  const int f0 = m0 / a.rows_per_signal, f1 = (m1 - 1) / a.rows_per_signal;
  const unsigned long long t0 = wall_clock64();
  enum : int { ARRIVED = 1, GIVE_UP = 2, HELP = 3, SELF_SERVE = 4 };
  const int nf = f1 - f0 + 1;
  // The search for a piece covers a window of at most 4096 pieces (12 index bits in the key below),
  // starting at the first tile whose signal is still missing, so it moves on as tiles complete.
  const int window_tiles = a.copy_pieces > 0 ? (4096 / a.copy_pieces < nf ? 4096 / a.copy_pieces : nf) : 0;
  uint32_t salt = (uint32_t)blockIdx.x * 0x9E3779B9u;      // varies per workgroup and per attempt
  int dead_w0 = -1;                                        // window start at which a search found nothing left to take
  bool ok = true;
  uint32_t call_id = 0u;                                   // fetched when a piece is first looked for
  bool have_call_id = false;
  for (;;) {
    if (tid < 64) {
      // the first wave polls, one signal per lane: one memory round trip per 64 signals, however
      // many the tile waits for (a decode tile waits for all of them)
      int st;
      int first_missing = 0;
      for (int polls = 0;; ++polls) {
        first_missing = -1;
        for (int base = 0; base < nf && first_missing < 0; base += 64) {
          const bool unset = base + tid < nf &&
                             __hip_atomic_load(a.signals + f0 + base + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == 0u;
          const unsigned long long missing = __ballot(unset);
          if (missing != 0) first_missing = f0 + base + __builtin_ctzll(missing);
        }
        if (first_missing < 0) { st = ARRIVED; break; }
        if (wall_clock64() - t0 > a.timeout_ticks) {
          if (tid == 0 && atomicCAS(a.status, 0u, (uint32_t)FLUX_ERR_TIMEOUT) == 0u) a.status[1] = (uint32_t)first_missing;
          st = GIVE_UP;
          break;
        }
        if (a.copy_pieces > 0 && first_missing != dead_w0 &&
            (a.copy_eager || (polls >= 8 && !driver_fully_started(a.started_counter, a.copy_driver_wgs)))) {
          st = HELP;
          break;
        }
        if (a.copy_pieces == 0 && a.self_serve_ticks != 0u && wall_clock64() - t0 > (unsigned long long)a.self_serve_ticks) {
          st = SELF_SERVE;
          break;
        }
        __builtin_amdgcn_s_sleep(16);
      }
      if (tid == 0) {
        lds[0] = st;
        lds[1] = 0x7fffffff;
        lds[3] = first_missing;
      }
    }
    __syncthreads();
    // (read as scalars: the compiler takes a value loaded from LDS for one that may differ between lanes,
    // and everything changed inside a loop left under such a value, like the transfer's cursors, with it)
    const int st = __builtin_amdgcn_readfirstlane(lds[0]);
    const int w0 = __builtin_amdgcn_readfirstlane(lds[3]);                // first tile of the search window
    __syncthreads();                    // everyone has read them before the first wave can write again
    if (st == ARRIVED) break;
    if (st == GIVE_UP) { ok = false; break; }
    if (st == SELF_SERVE) {
      // The transfers of a driver that takes no pieces (a library copy per tile with a stream write
      // of its signal) run as kernels of their own on this chip: when the grid's waiting workgroups
      // hold every compute unit, those kernels cannot start and the signals never come.  A workgroup
      // that has waited long enough therefore fetches the rows of its own tile from the chunk
      // sources itself and goes on without its signals.  The driver may write the same bytes to the
      // same places at the same time: harmless.  (The host puts the signals back after the join in
      // this form, since a driver that was overtaken sets some of them after the grid is done.)
      const unsigned long long vec_per_row = (unsigned long long)a.K / 8;
      const unsigned long long nvec = (unsigned long long)(m1 - m0) * vec_per_row;
      for (unsigned long long v = tid; v < nvec; v += 4 * blockDim.x) {
        u32x4 x[4];
        const uint4* src[4];
        uint4* dst[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const unsigned long long vv = v + (unsigned long long)u * blockDim.x;
          const int row = m0 + (int)((vv < nvec ? vv : 0) / vec_per_row);
          const unsigned long long col = (vv < nvec ? vv : 0) % vec_per_row;
          const int chunk = row / a.S;
          src[u] = static_cast<const uint4*>(lds_srcs[chunk]) + (unsigned long long)(row - chunk * a.S) * vec_per_row + col;
          dst[u] = reinterpret_cast<uint4*>(const_cast<__bf16*>(a.A)) + (unsigned long long)row * ((unsigned long long)a.lda / 8) + col;
          if (vv < nvec) x[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src[u]));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (v + (unsigned long long)u * blockDim.x < nvec && src[u] != dst[u]) store_through(dst[u], x[u]);
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): the stores are acknowledged
      __syncthreads();
      break;
    }
    // One of the unclaimed pieces among the tiles of the window, picked by a hash that differs per
    // workgroup and attempt: workgroups that wait for the same tiles then rarely go for the same
    // piece (taking "the first free one" would make them queue up behind each other).  The local
    // chunk's tiles are never copied by anyone, their signals are preset.
    if (!have_call_id) { call_id = transfer_call_id(a); have_call_id = true; }
    const int wt = f1 - w0 + 1 < window_tiles ? f1 - w0 + 1 : window_tiles;
    const int total = wt * a.copy_pieces;
    salt = salt * 1664525u + 1013904223u;
    for (int i = tid; i < total; i += blockDim.x) {
      const int f = w0 + i / a.copy_pieces;
      if (f >= a.sig_local_lo && f < a.sig_local_hi) continue;
      if (__hip_atomic_load(a.copy_claims + (size_t)f * a.copy_pieces + i % a.copy_pieces, __ATOMIC_RELAXED,
                            __HIP_MEMORY_SCOPE_AGENT) != call_id) {
        const uint32_t h = ((uint32_t)i * 2654435761u) ^ salt;
        atomicMin(&lds[1], (int)(((h >> 14) << 12) | (uint32_t)i));   // 18 hash bits above the 12-bit index: below the "none" value
      }
    }
    __syncthreads();
    const int key = lds[1];
    if (key != 0x7fffffff) {
      const int i = key & 4095;
      const int f = w0 + i / a.copy_pieces, piece = i % a.copy_pieces;
      if (tid == 0) lds[2] = claim_piece(a.copy_claims + (size_t)f * a.copy_pieces + piece, call_id) ? 1 : 0;
      __syncthreads();
      if (lds[2]) {
        const int ctpc = a.n_signals / a.R;
        const uint4* src = static_cast<const uint4*>(lds_srcs[f / ctpc]) + (unsigned long long)(f % ctpc) * a.copy_tile_vec;
        copy_piece(src, agg_tile(a, f), a.copy_tile_vec, piece, a.copy_pieces, tid, agg_pitch(a));
        finish_pieces(a.copy_counters + f, a.signals + f, a.copy_pieces, 1);
      }
    } else {
      dead_w0 = w0;                     // every piece of this window is in the hands of a workgroup that is running
    }
    __syncthreads();                    // lds[1], lds[2] are rewritten in the next round
  }
  if (tid == 0) {
    // Acquire.  The rows were written through to memory (write-through stores of a workgroup or of
    // the copy kernel, or a DMA engine) and acknowledged before their signal was set, and the poll
    // that saw the signal has returned, so loads issued from here on come after them.  What is
    // left to rule out is a stale copy in this die's L2 or this unit's L1.  Both are emptied when
    // a kernel starts, and nobody reads a row of the gathered matrix before its signal, so such a
    // copy can only exist if a cache line holds rows of two communication tiles.  Only then is
    // the die's L2 invalidated here: doing that costs one to two microseconds per workgroup and
    // throws out the operand panels the die's other workgroups are sharing.
    if (a.acquire_l2) __atomic_thread_fence(__ATOMIC_ACQUIRE);   // system scope
    else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    // count this workgroup in: its leaf first, the root if that completed the leaf
    const uint32_t leaf = blockIdx.x % DONE_LEAVES;
    const uint32_t quota = (gridDim.x - leaf + DONE_LEAVES - 1) / DONE_LEAVES;
    const uint32_t leaves = gridDim.x < (uint32_t)DONE_LEAVES ? gridDim.x : (uint32_t)DONE_LEAVES;
    uint32_t* leaf_counter = a.done_counter + (WS_DONELEAF_OFF - WS_DONE_OFF + leaf * DONE_LEAF_STRIDE) / 4;
    bool last = false;
    if (__hip_atomic_fetch_add(leaf_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == quota - 1) {
      __hip_atomic_store(leaf_counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
      last = __hip_atomic_fetch_add(a.done_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == leaves - 1;
    }
    if (last) {
      for (int i = 0; i < a.n_signals; ++i)
        __hip_atomic_store(a.signals + i, (i >= a.sig_local_lo && i < a.sig_local_hi) ? 1u : 0u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
      if (a.copy_pieces > 0 && a.copy_call_id == 0u)
        __hip_atomic_fetch_add(a.copy_call_seq, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (a.copy_driver_wgs > 0)
        __hip_atomic_fetch_add(a.started_counter + 1, (uint32_t)a.copy_driver_wgs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(a.done_counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
  return ok;
}

// Reduce by atomic additions on device memory (Sec. 4.2, "Reduce", first form): the owner's fp32 slice
// already holds what the other ranks have added; every element of the tile is added to it with one
// hardware addition that returns nothing.  The lanes of an instruction take consecutive columns of a
// row, so that an instruction touches two whole cache lines and not sixteen partial ones (with the
// eight-columns-per-lane layout of the other epilogues this form took five times as long).
template <class C, bool EDGE>
__device__ __forceinline__ void epilogue_all_atomic(const GemmArgs& a, void* const* lds_outs, float* ep, f32x16 (&acc)[C::MI][C::NI],
                                                    int m0, int n0, int lane, int wm, int wn) {
  constexpr int W = C::WTN < 64 ? C::WTN : 64;   // columns per instruction
  constexpr int RPI = 64 / W;                    // rows per instruction
  const int c_in = lane % W, r_in = lane / W;
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi) {
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        ep[r * C::EP_STRIDE + ni * 32 + (lane & 31)] = acc[mi][ni][e];
      }
    __builtin_amdgcn_wave_barrier();
    for (int r0 = 0; r0 < 32; r0 += RPI) {
      const int r = r0 + r_in;
      const int gm = m0 + wm * C::WTM + mi * 32 + r;
      const int owner = gm / a.S;
      float* row = static_cast<float*>(lds_outs[owner]) + (size_t)(gm - owner * a.S) * a.ldc + n0 + wn * C::WTN;
#pragma unroll
      for (int c0 = 0; c0 < C::WTN; c0 += W) {
        const int c = c0 + c_in;
        if (!EDGE || (gm < a.M && n0 + wn * C::WTN + c < a.N)) unsafeAtomicAdd(row + c, ep[r * C::EP_STRIDE + c]);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// Everything after the main loop: the split-K hand-over (all but the last-arriving workgroup of
// a tile park their partial sums, the last one adds them up) and the epilogue, in which the
// accumulators pass through LDS once (per wave, 32 rows at a time) so that every lane ends up
// with 8 consecutive columns of one row.  `smem` must hold C::EP_BYTES and is free to reuse.
template <class C, int EPI, bool EDGE>
__device__ __forceinline__ void gemm_tail(const GemmArgs& a, unsigned char* smem, int* lds_misc, void* const* lds_outs,
                                          f32x16 (&acc)[C::MI][C::NI], int tile, int split, bool is_split,
                                          int m0, int n0, int tid, int lane, int wave, int wm, int wn, int vb = -1) {
  trace_stamp(a, TRACE_MAIN_END, vb);
  // ---- split-K: all but the last-arriving workgroup of a tile park their partial sums ----
  if (is_split) {
    const int st = tile - a.full_tiles;            // index among the split tiles
    // Partials are stored and re-read with device-scope (sc1) accesses, which go through the
    // die's L2 to memory: the hand-over between workgroups on different dies then needs neither
    // an L2 write-back nor an L2 invalidate, only "my stores are acknowledged" before counting in.
    constexpr int SC1 = 16;                               // cache-policy bit: device scope
    constexpr int BLOCK_BYTES = C::BM * C::BN * 4;
    float* mine = a.sk_partials + ((size_t)split * a.split_tiles + st) * (C::BM * C::BN);
    __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(mine, 0, BLOCK_BYTES, 0x00027000);
    // layout inside a tile's partial block: [vector index][thread] -> coalesced 16-byte columns.
    // A vector holds four of eight consecutive rows; with a ragged M (a decode tile of 8 rows in a
    // 32-row tile) the vectors that lie wholly past the last row are neither parked nor read back:
    // their offset is moved past the end of the block, where the range check of the buffer drops a
    // store and answers a load with zeros (a branch around them would make every load wait for
    // the one before).
    const int rows_valid = EDGE ? a.M - m0 - wm * C::WTM : C::BM;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const u32x4 v = {__float_as_uint(acc[mi][ni][4 * q]), __float_as_uint(acc[mi][ni][4 * q + 1]),
                           __float_as_uint(acc[mi][ni][4 * q + 2]), __float_as_uint(acc[mi][ni][4 * q + 3])};
          const bool past = EDGE && mi * 32 + 8 * q >= rows_valid;
          __builtin_amdgcn_raw_buffer_store_b128(v, rm, past ? BLOCK_BYTES : (((mi * C::NI + ni) * 4 + q) * C::NT + tid) * 16, 0, SC1);
        }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0): stores acknowledged
    __syncthreads();
    int* lds_last = lds_misc;
    if (tid == 0) {
      const uint32_t prev = __hip_atomic_fetch_add(a.sk_counters + st, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int last = prev == (uint32_t)(a.split_k - 1);
      if (last) __hip_atomic_store(a.sk_counters + st, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
      *lds_last = last;
    }
    __syncthreads();
    trace_stamp(a, TRACE_END, vb);    // a workgroup that is not the tile's last ends here
    if (!*lds_last) return;
    // The sum always runs over the parked partials in split order, whichever workgroup happens
    // to be last, so results do not depend on arrival timing.  (Keeping the own part in registers
    // and skipping its load was tried: no gain for 64x64 tiles, a loss for 64x128.)
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.f;
    // Sixteen or thirty-two loads are issued before the first is used.  Left to itself the compiler waits for
    // every vector before it requests the next (a memory round trip each: 17 us for the 256 KB of
    // two parts of a 256x128 tile); a branch around a load has the same effect, so parts past the
    // end are read as zeros through the buffer's range check instead.  A large tile takes its
    // vectors a batch at a time, part by part; a small one takes all vectors of several parts.
    constexpr int NVEC = C::MI * C::NI * 4;                 // 16-byte vectors per thread and part
    constexpr int IN_FLIGHT = NVEC >= 32 ? 32 : 16;         // (32 is ahead for the large tiles, 16 for the small)
    constexpr int VB = NVEC < IN_FLIGHT ? NVEC : IN_FLIGHT; // vectors per batch within a part
    constexpr int PB = IN_FLIGHT / VB;                      // parts per batch
    static_assert(NVEC % VB == 0 && IN_FLIGHT % VB == 0, "batches divide the tile");
    for (int s0 = 0; s0 < a.split_k; s0 += PB) {
#pragma unroll
      for (int b0 = 0; b0 < NVEC; b0 += VB) {
        u32x4 v[PB][VB];
#pragma unroll
        for (int g = 0; g < PB; ++g) {
          const int s = s0 + g;
          const bool none = s >= a.split_k;                 // only with PB > 1
          float* other = a.sk_partials + ((size_t)(none ? 0 : s) * a.split_tiles + st) * (C::BM * C::BN);
          __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(other, 0, BLOCK_BYTES, 0x00027000);
#pragma unroll
          for (int i = 0; i < VB; ++i) {
            const int idx = b0 + i, mi = idx / (C::NI * 4), q = idx % 4;
            const bool past = none || (EDGE && mi * 32 + 8 * q >= rows_valid);
            v[g][i] = __builtin_amdgcn_raw_buffer_load_b128(ro, past ? BLOCK_BYTES : (idx * C::NT + tid) * 16, 0, SC1);
          }
        }
        __builtin_amdgcn_sched_barrier(0);                  // all of the batch's loads first
#pragma unroll
        for (int g = 0; g < PB; ++g)
#pragma unroll
          for (int i = 0; i < VB; ++i) {
            const int idx = b0 + i, mi = idx / (C::NI * 4), ni = (idx / 4) % C::NI, q = idx % 4;
            acc[mi][ni][4 * q] += __uint_as_float(v[g][i][0]);
            acc[mi][ni][4 * q + 1] += __uint_as_float(v[g][i][1]);
            acc[mi][ni][4 * q + 2] += __uint_as_float(v[g][i][2]);
            acc[mi][ni][4 * q + 3] += __uint_as_float(v[g][i][3]);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
  }

  // ---- epilogue: registers -> LDS (per wave, 32 rows at a time) -> 8 columns per lane ----
  float* ep = reinterpret_cast<float*>(smem) + wave * (32 * C::EP_STRIDE);
  // (the dtype and rank-count tests stay outside the loop over blocks: inside it, the accumulators
  // would no longer be kept in registers.  Up to 8 ranks, 7 peer loads per piece are issued, else 15:
  // loads from absent peers return zeros but still cost an issue slot and four registers each.)
  constexpr int NP_ALL = FLUX_MAX_RANKS - 1, NP_8 = 7;
  if (EPI == EPI_RS && a.write_only == 2) {
    epilogue_all_atomic<C, EDGE>(a, lds_outs, ep, acc, m0, n0, lane, wm, wn);
  } else if (EPI != EPI_RS || a.write_only) {
    epilogue_all<C, EPI, EDGE, false, 2, 0>(a, lds_outs, ep, acc, m0, n0, lane, wm, wn);
  } else if (a.R <= NP_8 + 1) {
    if (a.partial_f32) epilogue_all<C, EPI, EDGE, true, 1, NP_8>(a, lds_outs, ep, acc, m0, n0, lane, wm, wn);
    else epilogue_all<C, EPI, EDGE, false, 2, NP_8>(a, lds_outs, ep, acc, m0, n0, lane, wm, wn);
  } else {
    if (a.partial_f32) epilogue_all<C, EPI, EDGE, true, 1, NP_ALL>(a, lds_outs, ep, acc, m0, n0, lane, wm, wn);
    else epilogue_all<C, EPI, EDGE, false, 1, NP_ALL>(a, lds_outs, ep, acc, m0, n0, lane, wm, wn);
  }
  if (EPI == EPI_RS && a.tile_ready != nullptr) {
    // Producer side of the tile-ready handshake (Sec. 4.2, "Reduce", second form): the tile was written
    // through to memory; once every wave's stores are acknowledged, count this producer in.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (tid == 0)
      __hip_atomic_fetch_add(a.tile_ready + (size_t)(m0 / C::BM) * a.tm.tiles_n + n0 / C::BN, 1u, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_SYSTEM);
  }
  trace_stamp(a, TRACE_END, vb);
}

template <class C, int EPI, bool WAIT, bool EDGE>
__global__ void __launch_bounds__(C::NT, C::OCC) gemm_kernel(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;

  int tile, split;
  bool is_split;
  map_block(a, (int)blockIdx.x, tile, split, is_split);
  int mt, nt;
  tile_coord(a.tm, tile, mt, nt);
  const int m0 = mt * C::BM, n0 = nt * C::BN;
  const int m1 = m0 + C::BM < a.M ? m0 + C::BM : a.M;
  trace_begin(a, tile, mt, nt, split, is_split);

  // output slices by rank (reduce-scatter) or chunk sources by rank (all-gather)
  void** lds_outs = reinterpret_cast<void**>(smem + C::PTRS_OFF);
  if (EPI == EPI_RS || WAIT) {
    fill_lds_outs(a, lds_outs, tid);
  }

  if (WAIT) {
    transfer_own_pieces(a, reinterpret_cast<int*>(smem + C::MISC_OFF), lds_outs);
    if (!wait_signals(a, m0, m1, reinterpret_cast<int*>(smem + C::MISC_OFF), lds_outs)) { trace_stamp(a, TRACE_END); return; }
    trace_stamp(a, TRACE_READY);
  }

  const int k_begin = is_split ? split * a.k_per_split : 0;
  const int k_end = (is_split && k_begin + a.k_per_split < a.K) ? k_begin + a.k_per_split : a.K;
  const int KT = (k_end - k_begin + C::BK - 1) / C::BK;

  f32x16 acc[C::MI][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.f;

  Loader<C, EDGE> ld;
  ld.init(a, m0, n0, tid);
  uint4 ra[C::A_VEC], rb[C::B_VEC];

  if (KT > 0) {
    ld.load(a, k_begin, k_end, ra, rb);
    ld.store(smem, ra, rb);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
      unsigned char* cur = smem + (C::ESTAGE == 2 ? (kt & 1) * C::STAGE_BYTES : 0);
      const bool more = kt + 1 < KT;
      if (more) ld.load(a, k_begin + (kt + 1) * C::BK, k_end, ra, rb);
      mma_stage<C>(cur, wm, wn, lane, acc);
      if (C::ESTAGE == 1) __syncthreads();
      if (more) ld.store(smem + (C::ESTAGE == 2 ? ((kt + 1) & 1) * C::STAGE_BYTES : 0), ra, rb);
      __syncthreads();
    }
  }

  gemm_tail<C, EPI, EDGE>(a, smem, reinterpret_cast<int*>(smem + C::MISC_OFF), lds_outs, acc, tile, split, is_split,
                          m0, n0, tid, lane, wave, wm, wn);
}


// ---------------------------------------------------------------------------------------------
// Fast path for shapes that the tile divides: global -> LDS without passing through registers.
//
// buffer_load_dwordx4 ... lds writes the 64 x 16 B a wave fetches to 1 KiB of consecutive LDS,
// so the swizzled layouts above are produced by permuting which 16 B each lane FETCHES:
//   A: one instruction = 8 rows x 128 B; lane i fills physical slot i%8 of row i/8 and fetches
//      logical slot (i%8) ^ swz_a(row);
//   B: one instruction = 1 KiB / (2*BN) k-rows; lane i fills physical slot i%B_SLOTS and
//      fetches logical slot (i%B_SLOTS) ^ swz_b(k).
// Per K-slab only scalar offsets change (soffset), so the address arithmetic costs no vector
// instructions.  The two LDS stages are separate arrays: the compiler's wait-count insertion can
// then tell the stage being filled from the stage being read and does not serialise them.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void_t;

template <class C>
struct DmaLoader {
  static constexpr int NW = C::NT / 64;
  static constexpr int A_RPI = 8;                              // A rows per instruction (1 KiB of 128-byte rows)
  static constexpr int A_INSTR = C::BM / A_RPI / NW;           // per wave
  static constexpr int RPI = C::B_NK ? A_RPI : 512 / C::BN;    // B rows per instruction: k-rows of BN values, or ([N,K]) n-rows of BK
  static constexpr int B_INSTR = (C::B_NK ? C::BN : C::BK) / RPI / NW;   // per wave
  static_assert(C::BK == 64, "A rows must be 128 B");
  static_assert(NW % 2 == 0 && (RPI * NW) % 4 == 0, "swizzle must not depend on the instruction index");
  static_assert(C::BM % (A_RPI * NW) == 0 && (C::B_NK ? C::BN : C::BK) % (RPI * NW) == 0 && 512 % C::BN == 0, "loader shape");

  // Offsets into A and B are unsigned 32-bit byte offsets (a matrix has fewer than 2^31 elements, so
  // fewer than 2^32 bytes); the hardware adds the vector and the scalar part as unsigned numbers.
  __amdgpu_buffer_rsrc_t ra, rb;
  uint32_t voff_a, voff_b;
  uint32_t K2, N2;               // row pitches in bytes

  __device__ __forceinline__ void init(const GemmArgs& a, int m0, int n0, int wave, int lane) {
    ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(a.A), 0, (int)(((unsigned)(a.M - 1) * (unsigned)a.lda + (unsigned)a.K) * 2u), 0x00027000);
    rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(a.B), 0,
                                           (int)((C::B_NK ? (unsigned)(a.N - 1) * (unsigned)a.ldb + (unsigned)a.K
                                                          : (unsigned)(a.K - 1) * (unsigned)a.ldb + (unsigned)a.N) * 2u), 0x00027000);
    const int r_in = lane / C::A_SLOTS, sp = lane % C::A_SLOTS;
    const int row = A_RPI * wave + r_in;
    K2 = (uint32_t)a.lda * 2u;
    N2 = (uint32_t)a.ldb * 2u;
    voff_a = (uint32_t)(m0 + row) * K2 + ((uint32_t)(sp ^ swz_a<C::A_SLOTS>(row)) << 4);
    if constexpr (C::B_NK) {
      voff_b = (uint32_t)(n0 + row) * N2 + ((uint32_t)(sp ^ swz_a<C::A_SLOTS>(row)) << 4);      // as for A, rows of n
    } else {
      const int k_in = lane / C::B_SLOTS, spb = lane % C::B_SLOTS;
      const int k = RPI * wave + k_in;
      voff_b = (uint32_t)k * N2 + (uint32_t)n0 * 2u + ((uint32_t)(spb ^ swz_b<C::B_SLOTS>(k)) << 4);
    }
  }
  static constexpr int N_INSTR = A_INSTR + B_INSTR;

  // same with an index that is constant after loop unrolling
  __device__ __forceinline__ void issue_dyn(int idx, const GemmArgs& a, unsigned char* stage, int k0, int wave) const {
    if (idx < A_INSTR) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void_t*)(stage + (idx * NW + wave) * 1024), 16, (int)voff_a,
                                               (int)((uint32_t)k0 * 2u + (uint32_t)(idx * A_RPI * NW) * K2), 0, 0);
    } else {
      const int p = idx - A_INSTR;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void_t*)(stage + C::A_BYTES + (p * NW + wave) * 1024), 16, (int)voff_b,
                                               (int)(C::B_NK ? (uint32_t)k0 * 2u + (uint32_t)(p * RPI * NW) * N2 : (uint32_t)(k0 + p * RPI * NW) * N2), 0, 0);
    }
  }

  // this wave's loads of the A part / the B part of one K-slab; `stage` is the base of the LDS stage being filled
  __device__ __forceinline__ void issue_a(const GemmArgs& a, unsigned char* stage, int k0, int wave) const {
#pragma unroll
    for (int p = 0; p < A_INSTR; ++p)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void_t*)(stage + (p * NW + wave) * 1024), 16, (int)voff_a,
                                               (int)((uint32_t)k0 * 2u + (uint32_t)(p * A_RPI * NW) * K2), 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  __device__ __forceinline__ void issue_b(const GemmArgs& a, unsigned char* stage, int k0, int wave) const {
#pragma unroll
    for (int p = 0; p < B_INSTR; ++p)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void_t*)(stage + C::A_BYTES + (p * NW + wave) * 1024), 16, (int)voff_b,
                                               (int)(C::B_NK ? (uint32_t)k0 * 2u + (uint32_t)(p * RPI * NW) * N2 : (uint32_t)(k0 + p * RPI * NW) * N2), 0, 0);
    // keep the loads where they are written: scheduled late they would be issued just before
    // the wait for them, and nothing would overlap
    __builtin_amdgcn_sched_barrier(0);
  }
  // all loads of one K-slab for this wave
  __device__ __forceinline__ void issue(const GemmArgs& a, unsigned char* stage, int k0, int wave) const {
    issue_a(a, stage, k0, wave);
    issue_b(a, stage, k0, wave);
  }
};

template <class C>
__device__ __forceinline__ bf16x8 frag_a(const unsigned char* stage, int ks, int mi, int wm, int lane) {
  const int row = wm * C::WTM + mi * 32 + (lane & 31);
  const int q = ks * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(stage + row * (C::BK * 2) + ((q ^ swz_a<C::A_SLOTS>(row)) << 4));
}

template <class C>
__device__ __forceinline__ bf16x8 frag_b(const unsigned char* stage, int ks, int ni, int wn, int lane) {
  if constexpr (C::B_NK) {
    const int row = wn * C::WTN + ni * 32 + (lane & 31);
    const int q = ks * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(stage + C::A_BYTES + row * (C::BK * 2) + ((q ^ swz_a<C::A_SLOTS>(row)) << 4));
  }
  const int g = lane >> 4, i = lane & 15;
  const int k = ks * 16 + 8 * (g >> 1) + (i >> 2);
  const int n = wn * C::WTN + ni * 32 + 16 * (g & 1) + 4 * (i & 3);
  const int off = C::A_BYTES + k * (C::BN * 2) + ((((n >> 3) ^ swz_b<C::B_SLOTS>(k))) << 4) + ((n >> 2) & 1) * 8;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(stage + off));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(stage + off + 4 * C::BN * 2));
  s16x8 w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, w);
}

// The same two fragment reads as instructions the compiler cannot look into.  For every LDS read
// it can see, the compiler works out by itself how many of the direct-to-LDS loads still in flight
// must land first; around a ring of more than two stages it gets that wrong on the safe side and
// drains the pipeline.  With these reads the waits are the kernel's own: the counter wait before
// the workgroup barrier for the loads, wait_lds_reads() for the fragments.
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
__device__ __forceinline__ uint32_t lds_address(const unsigned char* p) {
  return (uint32_t)reinterpret_cast<uintptr_t>((const lds_byte_t*)p);
}

template <class C>
__device__ __forceinline__ bf16x8 frag_a_opaque(uint32_t stage, int ks, int mi, int wm, int lane) {
  const int row = wm * C::WTM + mi * 32 + (lane & 31);
  const int q = ks * 2 + (lane >> 5);
  const uint32_t addr = stage + row * (C::BK * 2) + ((q ^ swz_a<C::A_SLOTS>(row)) << 4);
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return __builtin_bit_cast(bf16x8, v);
}

template <class C>
__device__ __forceinline__ bf16x8 frag_b_opaque(uint32_t stage, int ks, int ni, int wn, int lane) {
  if constexpr (C::B_NK) {
    const int row = wn * C::WTN + ni * 32 + (lane & 31);
    const int q = ks * 2 + (lane >> 5);
    const uint32_t addr = stage + C::A_BYTES + row * (C::BK * 2) + ((q ^ swz_a<C::A_SLOTS>(row)) << 4);
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return __builtin_bit_cast(bf16x8, v);
  }
  const int g = lane >> 4, i = lane & 15;
  const int k = ks * 16 + 8 * (g >> 1) + (i >> 2);
  const int n = wn * C::WTN + ni * 32 + 16 * (g & 1) + 4 * (i & 3);
  const uint32_t addr = stage + C::A_BYTES + k * (C::BN * 2) + ((((n >> 3) ^ swz_b<C::B_SLOTS>(k))) << 4) + ((n >> 2) & 1) * 8;
  typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
  u32x2 lo, hi;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr) : "memory");
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(hi) : "v"(addr + 4 * C::BN * 2) : "memory");
  const u32x4 w = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, w);
}

// All LDS reads issued so far have returned.  The fragments pass through it so that nothing that
// uses them can be moved in front of the wait.
template <int MI, int NI>
__device__ __forceinline__ void wait_lds_reads(bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < MI; ++i) asm volatile("" : "+v"(af[i]));
#pragma unroll
  for (int i = 0; i < NI; ++i) asm volatile("" : "+v"(bfr[i]));
}

// One K-slab out of LDS stage `cur`, software-pipelined by hand:
//   * the MFMAs run in (ks, mi) groups of NI; the fragments of k-step ks+1 are fetched while the
//     MFMAs of ks run (two register sets);
//   * the wave's DMA loads for the NEXT slab (into `nxt`) are dealt out one group at a time.  A
//     wave issues in order, and a burst of loads would hold it in the memory pipeline's queue
//     for about as long as the slab's MFMAs take; spread out, the loads drain behind the MFMAs.
// Loads are only placed in the first SPREAD_NUM/SPREAD_DEN of the groups so the last one has
// time to land before the end-of-slab wait.
template <class C, bool ISSUE>
__device__ __forceinline__ void mma_stage_dma(const unsigned char* cur, unsigned char* nxt, const DmaLoader<C>& ld,
                                              const GemmArgs& a, int k_next, int wave, int wm, int wn, int lane,
                                              f32x16 (&acc)[C::MI][C::NI]) {
  constexpr int KS = C::BK / 16;
  constexpr int G = KS * C::MI;                       // MFMA groups in the slab
  constexpr int L = DmaLoader<C>::N_INSTR;            // loads to place
  constexpr int GS = (G * 3 + 3) / 4;                 // groups that carry loads
  // (the slab's offset goes into the loads' scalar operand: should the compiler ever take the loop
  // counter for a value that may differ between lanes, it would wrap every load into a loop over lanes)
  k_next = __builtin_amdgcn_readfirstlane(k_next);
  bf16x8 af[2][C::MI], bfr[2][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi) af[0][mi] = frag_a<C>(cur, 0, mi, wm, lane);
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) bfr[0][ni] = frag_b<C>(cur, 0, ni, wn, lane);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
      const int g = ks * C::MI + mi;
      // loads [g*L/GS, (g+1)*L/GS) go with group g (compile-time after unrolling)
      if (ISSUE && g < GS) {
        const int lo = g * L / GS, hi = (g + 1) * L / GS;
#pragma unroll
        for (int idx = 0; idx < L; ++idx)
          if (idx >= lo && idx < hi) ld.issue_dyn(idx, a, nxt, k_next, wave);
      }
      if (mi == 0 && ks + 1 < KS) {
#pragma unroll
        for (int m2 = 0; m2 < C::MI; ++m2) af[(ks + 1) & 1][m2] = frag_a<C>(cur, ks + 1, m2, wm, lane);
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni) bfr[(ks + 1) & 1][ni] = frag_b<C>(cur, ks + 1, ni, wn, lane);
      }
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][mi], bfr[ks & 1][ni], acc[mi][ni], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// mma_stage_dma with the opaque fragment reads: the fragments of k-step ks are waited for at the
// top of the step, then those of ks+1 are requested, then the MFMAs of ks run.
template <class C>
__device__ __forceinline__ void mma_stage_dma_opaque(const unsigned char* cur_p, unsigned char* nxt, const DmaLoader<C>& ld,
                                                     const GemmArgs& a, int k_next, int wave, int wm, int wn, int lane,
                                                     f32x16 (&acc)[C::MI][C::NI]) {
  constexpr int KS = C::BK / 16;
  constexpr int G = KS * C::MI;
  constexpr int L = DmaLoader<C>::N_INSTR;
  constexpr int GS = (G * 3 + 3) / 4;
  const uint32_t cur = lds_address(cur_p);
  if constexpr (C::MI * C::NI <= 2) {
    // One or two MFMAs per k-step (the 32x32 and 32x64 wave tiles of the few-row configurations):
    // too little to hide a k-step's fragment reads behind, so reading step by step pays the LDS
    // latency four times per slab.  Request the next slab first, fetch all fragments of this one in
    // one go (48 registers at most), wait once.
    ld.issue(a, nxt, k_next, wave);
    bf16x8 af[KS * C::MI], bfr[KS * C::NI];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi) af[ks * C::MI + mi] = frag_a_opaque<C>(cur, ks, mi, wm, lane);
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni) bfr[ks * C::NI + ni] = frag_b_opaque<C>(cur, ks, ni, wn, lane);
    }
    wait_lds_reads<KS * C::MI, KS * C::NI>(af, bfr);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks * C::MI + mi], bfr[ks * C::NI + ni], acc[mi][ni], 0, 0, 0);
    return;
  }
  bf16x8 af[2][C::MI], bfr[2][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi) af[0][mi] = frag_a_opaque<C>(cur, 0, mi, wm, lane);
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) bfr[0][ni] = frag_b_opaque<C>(cur, 0, ni, wn, lane);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    wait_lds_reads<C::MI, C::NI>(af[ks & 1], bfr[ks & 1]);
    if (ks + 1 < KS) {
#pragma unroll
      for (int m2 = 0; m2 < C::MI; ++m2) af[(ks + 1) & 1][m2] = frag_a_opaque<C>(cur, ks + 1, m2, wm, lane);
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni) bfr[(ks + 1) & 1][ni] = frag_b_opaque<C>(cur, ks + 1, ni, wn, lane);
    }
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
      const int g = ks * C::MI + mi;
      if (g < GS) {
        const int lo = g * L / GS, hi = (g + 1) * L / GS;
#pragma unroll
        for (int idx = 0; idx < L; ++idx)
          if (idx >= lo && idx < hi) ld.issue_dyn(idx, a, nxt, k_next, wave);
      }
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][mi], bfr[ks & 1][ni], acc[mi][ni], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

template <int N>
__device__ __forceinline__ void wait_vm_at_most() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));   // expcnt and lgkmcnt: no wait
}

// Workgroup barrier that lets this wave's younger loads stay in flight.  The compiler puts a wait
// for ALL outstanding memory operations in front of every barrier instruction it can see, which
// would empty the pipeline once per slab; it does not look inside this one.  What the barrier has
// to order is covered by the counter wait placed before it.
__device__ __forceinline__ void barrier_keeping_loads_in_flight() {
  asm volatile("s_barrier" ::: "memory");
}

__device__ __forceinline__ void wait_vm0_and_barrier() {
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's LDS-bound loads have landed
  __syncthreads();
}

template <class C, int EPI, bool WAIT>
__global__ void __launch_bounds__(C::NT, C::OCC) gemm_kernel_dma(const GemmArgs a) {
  constexpr int S0_BYTES = C::STAGE_BYTES > C::EP_BYTES ? C::STAGE_BYTES : C::EP_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char stage0[S0_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char stage1[C::STAGE_BYTES];
  __shared__ int lds_misc[4];
  __shared__ void* lds_outs[FLUX_MAX_RANKS];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;

  int tile, split;
  bool is_split;
  map_block(a, (int)blockIdx.x, tile, split, is_split);
  int mt, nt;
  tile_coord(a.tm, tile, mt, nt);
  const int m0 = mt * C::BM, n0 = nt * C::BN;
  trace_begin(a, tile, mt, nt, split, is_split);

  if (EPI == EPI_RS || WAIT) {      // output slices (reduce-scatter) or chunk sources (all-gather), by rank
    fill_lds_outs(a, lds_outs, tid);
  }
  SideCopy side;
  if (WAIT) {
    transfer_own_pieces(a, lds_misc, lds_outs);
    side.begin(a, lds_misc + 2, lds_outs);     // (also orders fill_lds_outs before the reads of lds_outs below)
    // A workgroup that has pieces to move and no data to compute on yet moves them in batches, and
    // counts tiles in as they become due, until its own signals are there (the main loop then
    // carries what is left) or its part of the transfer is done (then it waits like anybody else).
    while (side.pending() && !signals_all_set(a, m0, m0 + C::BM, lds_misc + 2)) {
      if (!side.all_stored()) side.pump(a, lds_outs);
      else __builtin_amdgcn_s_sleep(16);
      side.maybe_finish(a);
    }
    if (!wait_signals(a, m0, m0 + C::BM, lds_misc, lds_outs)) {
      // given up (a workgroup only gets to its wait with pieces left if its signals were there, so this
      // is for safety): the pieces it claimed still have to be moved, or their tiles' signals never come
      if (side.pending()) side.drain(a, lds_outs);
      trace_stamp(a, TRACE_END);
      return;
    }
    trace_stamp(a, TRACE_READY);
  }
  const int k_begin = is_split ? split * a.k_per_split : 0;
  const int k_end = (is_split && k_begin + a.k_per_split < a.K) ? k_begin + a.k_per_split : a.K;
  const int KT = (k_end - k_begin) / C::BK;

  f32x16 acc[C::MI][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.f;

  DmaLoader<C> ld;
  ld.init(a, m0, n0, wave, lane);
  ld.issue(a, stage0, k_begin, wave);
  wait_vm0_and_barrier();
  // Every slab prefetches its successor; the last one fetches itself again (into the stage that
  // is not being read), which keeps a single code shape for the loop instead of a prefetch-free
  // copy of it that the register allocator handles badly.
  const int k_last = k_begin + (KT - 1) * C::BK;
  int kt = 0;
  if (WAIT && side.pending()) {
    // With the transfer aboard (a workgroup of the first round with pieces to move; everybody else
    // runs the plain loop below): per slab two stores (of the vectors loaded two slabs ago) ahead of
    // the slab's operand loads and two loads behind them.  "All but the two youngest operations have
    // completed" then means that the operand loads have landed (loads complete in order, and the
    // stores are older than all of them), and the barrier must not make the compiler wait for those
    // last loads.  Thread 0 looks at the clock once per two slabs and leaves word in LDS whether a
    // tile is due to be counted in (a decision every wave must take alike: finish() has barriers).
    // When the last tile is counted in, the plain loop takes over for the rest of K.
    u32x4 dA0 = side.load(a, lds_outs), dA1 = side.load(a, lds_outs);
    u32x4 dB0 = side.load(a, lds_outs), dB1 = side.load(a, lds_outs);
    for (; kt + 2 <= KT && side.pending(); kt += 2) {
      side.store(a, dA0);
      side.store(a, dA1);
      mma_stage_dma<C, true>(stage0, stage1, ld, a, k_begin + (kt + 1) * C::BK, wave, wm, wn, lane, acc);
      dA0 = side.load(a, lds_outs);
      dA1 = side.load(a, lds_outs);
      wait_vm_at_most<2>();
      barrier_keeping_loads_in_flight();
      side.store(a, dB0);
      side.store(a, dB1);
      const int k2 = k_begin + (kt + 2) * C::BK;
      mma_stage_dma<C, true>(stage1, stage0, ld, a, k2 < k_last ? k2 : k_last, wave, wm, wn, lane, acc);
      dB0 = side.load(a, lds_outs);
      dB1 = side.load(a, lds_outs);
      const bool look = side.may_be_due();       // (uniform)
      if (look && tid == 0) *side.slot = side.due() ? 1 : 0;
      wait_vm_at_most<2>();
      barrier_keeping_loads_in_flight();
      if (look) {
        const int go = __builtin_amdgcn_readfirstlane(*side.slot);
        if (go) side.finish(a);           // (its barriers also keep the slot from being rewritten too early)
      }
    }
    wait_vm0_and_barrier();
    if (side.pending()) {          // K is over before the transfer is: the vectors in flight first, then the rest
      side.store(a, dA0); side.store(a, dA1); side.store(a, dB0); side.store(a, dB1);
      side.ld_t = side.st_t; side.ld_s = side.st_s; side.ld_off = side.st_off;     // the loads start again where the stores are
      side.set_src(a, lds_outs, side.ld_t);
      side.drain(a, lds_outs);
    }
  }
  for (; kt + 2 <= KT; kt += 2) {
    mma_stage_dma<C, true>(stage0, stage1, ld, a, k_begin + (kt + 1) * C::BK, wave, wm, wn, lane, acc);
    wait_vm0_and_barrier();
    const int k2 = k_begin + (kt + 2) * C::BK;
    mma_stage_dma<C, true>(stage1, stage0, ld, a, k2 < k_last ? k2 : k_last, wave, wm, wn, lane, acc);
    wait_vm0_and_barrier();
  }
  if (kt < KT) {
    mma_stage_dma<C, true>(stage0, stage1, ld, a, k_last, wave, wm, wn, lane, acc);
    wait_vm0_and_barrier();
  }
  gemm_tail<C, EPI, false>(a, stage0, lds_misc, lds_outs, acc, tile, split, is_split, m0, n0, tid, lane, wave, wm, wn);
}

// The same kernel as a grid of resident workgroups, one per compute unit, each walking the block
// sequence with the grid's stride (block b, b + grid, ...: the order of Sec. 4.1 is kept, in time
// instead of in dispatch).
template <class C, int EPI>
__global__ void __launch_bounds__(C::NT, C::OCC) gemm_kernel_dma_resident(const GemmArgs a_) {
  constexpr int S0_BYTES = C::STAGE_BYTES > C::EP_BYTES ? C::STAGE_BYTES : C::EP_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char stage0[S0_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char stage1[C::STAGE_BYTES];
  __shared__ int lds_misc[4];
  __shared__ void* lds_outs[FLUX_MAX_RANKS];
  if (EPI == EPI_RS) fill_lds_outs(a_, lds_outs, (int)threadIdx.x);
  if (a_.persist_delay_ticks != 0 && ((blockIdx.x >> 3) & 1)) {
    const uint64_t t0 = wall_clock64();
    while (wall_clock64() - t0 < a_.persist_delay_ticks) __builtin_amdgcn_s_sleep(32);
  }
  const int n_blocks = a_.persist_blocks;
  for (int vb = (int)blockIdx.x; vb < n_blocks; vb += (int)gridDim.x) {
    // The argument block is read afresh for every block (the struct is the kernel's only argument and
    // lies at the start of the argument segment): fetched once before the loop, its hundred-odd scalars
    // would be kept in registers across the main loop, which has none to spare.
    typedef const GemmArgs __attribute__((address_space(4))) * ArgPtr;
    ArgPtr ap = (ArgPtr)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
    const GemmArgs& a = *(const GemmArgs*)ap;
    // ... and so is everything a lane derives from its index (fragment addresses, load offsets)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    int tile, split;
    bool is_split;
    map_block(a, vb, tile, split, is_split);
    int mt, nt;
    tile_coord(a.tm, tile, mt, nt);
    const int m0 = mt * C::BM, n0 = nt * C::BN;
    trace_begin(a, tile, mt, nt, split, is_split, vb);
    const int k_begin = is_split ? split * a.k_per_split : 0;
    const int k_end = (is_split && k_begin + a.k_per_split < a.K) ? k_begin + a.k_per_split : a.K;
    const int KT = (k_end - k_begin) / C::BK;
    f32x16 acc[C::MI][C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.f;
    DmaLoader<C> ld;
    ld.init(a, m0, n0, wave, lane);
    ld.issue(a, stage0, k_begin, wave);
    wait_vm0_and_barrier();
    const int k_last = k_begin + (KT - 1) * C::BK;
    int kt = 0;
    for (; kt + 2 <= KT; kt += 2) {
      mma_stage_dma<C, true>(stage0, stage1, ld, a, k_begin + (kt + 1) * C::BK, wave, wm, wn, lane, acc);
      wait_vm0_and_barrier();
      const int k2 = k_begin + (kt + 2) * C::BK;
      mma_stage_dma<C, true>(stage1, stage0, ld, a, k2 < k_last ? k2 : k_last, wave, wm, wn, lane, acc);
      wait_vm0_and_barrier();
    }
    if (kt < KT) {
      mma_stage_dma<C, true>(stage0, stage1, ld, a, k_last, wave, wm, wn, lane, acc);
      wait_vm0_and_barrier();
    }
    gemm_tail<C, EPI, false>(a, stage0, lds_misc, lds_outs, acc, tile, split, is_split, m0, n0, tid, lane, wave, wm, wn, vb);
    __syncthreads();      // the staging area and lds_misc are the next block's
  }
}

// ---------------------------------------------------------------------------------------------
// The same pipeline with NSTAGE >= 3 LDS stages, for tiles that have little arithmetic per byte
// (few rows: decode).  Such a tile is bound by how many bytes its compute unit keeps in flight:
// slab kt is computed while the loads of slabs kt+1 .. kt+NSTAGE-1 are outstanding.  Loads land in
// issue order, so "all but the (NSTAGE-2) youngest slabs have landed" is a plain counter wait.
// Stages are separate arrays (see above); the epilogue has its own staging area, so the tail of
// the load pipeline need not drain before it starts.
// ---------------------------------------------------------------------------------------------
// MASK: M is not a multiple of the tile height.  Rows past M are read as zeros (they lie outside
// the buffer resource of A) and the epilogue leaves them out.
// Counter wait of the first pass of the deep pipeline when the weights' part of the first slabs
// was issued ahead of everything else: before slab j is read, at most the A parts of the slabs
// after it (up to slab NS-2) and the j whole slabs issued since may be outstanding.  `j` is a
// constant after unrolling; the wait instruction needs its count as an immediate.
template <int NS, int LA, int L, int J = 0>
struct FirstPassWait {
  static __device__ __forceinline__ void run(int j) {
    if constexpr (J < NS - 1) {
      if (j == J) wait_vm_at_most<(NS - 2 - J) * LA + J * L>();
      else FirstPassWait<NS, LA, L, J + 1>::run(j);
    }
  }
};

template <class C, int EPI, bool WAIT, bool MASK>
__global__ void __launch_bounds__(C::NT, C::OCC) gemm_kernel_dma_deep(const GemmArgs a) {
  constexpr int NS = C::NSTAGE;
  static_assert(NS >= 3 && NS <= 9, "3 to 9 stages");
  constexpr int L = DmaLoader<C>::N_INSTR;                  // loads per slab and wave
  static_assert((NS - 2) * L < 64, "outstanding loads must fit the counter");
  // One pool: the stages, and over them (once the main loop is done) the epilogue's staging area.
  constexpr int POOL_BYTES = NS * C::STAGE_BYTES > C::EP_BYTES ? NS * C::STAGE_BYTES : C::EP_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char pool[POOL_BYTES];
  __shared__ int lds_misc[4];
  __shared__ void* lds_outs[FLUX_MAX_RANKS];
  unsigned char* st[NS];
#pragma unroll
  for (int j = 0; j < NS; ++j) st[j] = pool + j * C::STAGE_BYTES;
  unsigned char* const ep_stage = pool;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;

  int tile, split;
  bool is_split;
  map_block(a, (int)blockIdx.x, tile, split, is_split);
  int mt, nt;
  tile_coord(a.tm, tile, mt, nt);
  const int m0 = mt * C::BM, n0 = nt * C::BN;
  trace_begin(a, tile, mt, nt, split, is_split);

  if (EPI == EPI_RS || WAIT) {
    fill_lds_outs(a, lds_outs, tid);
  }
  const int k_begin = is_split ? split * a.k_per_split : 0;
  const int k_end = (is_split && k_begin + a.k_per_split < a.K) ? k_begin + a.k_per_split : a.K;
  const int KT = (k_end - k_begin) / C::BK;

  DmaLoader<C> ld;
  ld.init(a, m0, n0, wave, lane);
  // Slabs past the end are replaced by the last one: every step issues the same number of loads,
  // which keeps the counter wait a constant and the loop one shape.  Such a repeat lands in a
  // stage whose slab has been consumed, never in the one the last slab is read from.
  const int last = KT - 1;
  constexpr int LA = DmaLoader<C>::A_INSTR;
  if (WAIT) {
    // First this workgroup's own pieces of the chunks: the whole grid waits for them.  Then the
    // weights, which do not depend on the gathered rows: their part of the first slabs is on its
    // way while the workgroup waits for its signals.  In the first pass of the loop the order of
    // issue is then [B of slabs 0..NS-2][A of slabs 0..NS-2][slab NS-1]..., and "slab j has landed"
    // means that at most the A parts after it and j whole slabs are out.
    transfer_own_pieces(a, lds_misc, lds_outs);
#pragma unroll
    for (int j = 0; j < NS - 1; ++j) ld.issue_b(a, st[j], k_begin + (j < last ? j : last) * C::BK, wave);
    const int m1 = (!MASK || m0 + C::BM < a.M) ? m0 + C::BM : a.M;
    if (!wait_signals(a, m0, m1, lds_misc, lds_outs)) {
      wait_vm_at_most<0>();        // nothing of this workgroup is left in flight towards its LDS
      trace_stamp(a, TRACE_END);
      return;
    }
    trace_stamp(a, TRACE_READY);
#pragma unroll
    for (int j = 0; j < NS - 1; ++j) ld.issue_a(a, st[j], k_begin + (j < last ? j : last) * C::BK, wave);
  } else {
#pragma unroll
    for (int j = 0; j < NS - 1; ++j) ld.issue(a, st[j], k_begin + (j < last ? j : last) * C::BK, wave);
  }

  f32x16 acc[C::MI][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.f;

  for (int kt0 = 0; kt0 < KT; kt0 += NS) {
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const int kt = kt0 + j;
      if (kt < KT) {
        // slab kt has landed (this wave's part of it)
        if (WAIT && j < NS - 1 && kt0 == 0) FirstPassWait<NS, LA, L>::run(j);
        else wait_vm_at_most<(NS - 2) * L>();
        barrier_keeping_loads_in_flight();   // ... everyone's part; and slab kt-1 has been read by all
        const int kn = kt + NS - 1 < last ? kt + NS - 1 : last;
        mma_stage_dma_opaque<C>(st[j], st[(j + NS - 1) % NS], ld, a, k_begin + kn * C::BK, wave, wm, wn, lane, acc);
      }
    }
  }
  wait_vm_at_most<0>();
  __syncthreads();       // the epilogue's staging area lies over stages other waves may still be reading
  gemm_tail<C, EPI, MASK>(a, ep_stage, lds_misc, lds_outs, acc, tile, split, is_split, m0, n0, tid, lane, wave, wm, wn);
}

}  // namespace flux
