/*
 * flux.h - C ABI of the MI355X (gfx950) library for tensor-parallel GEMMs with the
 * communication fused in at tile granularity.
 *
 * Two operations are covered, both seen from ONE rank of an N_TP-way tensor-parallel group
 * ("R virtual ranks": every peer buffer is a pointer into this GPU's own memory):
 *
 *   GEMM-ReduceScatter  (paper Alg. 1, Sec. 3.1, Sec. 4.1, Sec. 4.2 "Reduce")
 *       out[r][i - r*S, n] = cvt( sum_k A[i,k] B[k,n]  +  sum_{j != rank} peer_j[i,n] ),
 *       r = i / S, S = M / R.   One kernel: the reduction and the scatter to the owning
 *       rank's row slice happen in the GEMM epilogue; tiles are visited slice by slice
 *       starting after the local rank (rank-shifted TileCoord).
 *
 *   AllGather-GEMM      (paper Alg. 2 + Alg. 3 pull form, Sec. 3.2, Sec. 4.1, Sec. 4.3)
 *       C = A_agg B,  A_agg = rows of chunk 0, chunk 1, ... chunk R-1.
 *       A copy driver on `copy_stream` moves the remote chunks into A_agg in `arrival_order`
 *       and sets one 32-bit signal per communication tile; the GEMM kernel on
 *       `compute_stream` visits tiles in the same order and spins on the signals of the rows
 *       a tile needs before touching them (WaitSignal in the prologue).
 *
 * plus the non-overlapped baseline used for the overlap-efficiency metric (Sec. 2.3, Eq. 1-2).
 *
 * Conventions
 *   - All matrices are row-major: A [M,K], B [K,N] (or [N,K], see b_is_nk), partials / C [M,N], slices [M/R,N]; densely
 *     packed unless the problem gives a row pitch (lda / ldb / ldc of flux_problem_t, which also says
 *     which matrices each applies to).  A and B are bf16; partials and outputs are bf16 or f32
 *     (flux_dtype_t).
 *   - M % R == 0; N % 8 == 0; K % 8 == 0; every base pointer 16-byte aligned; R <= FLUX_MAX_RANKS.
 *   - Every pointer marked "device" must be device memory of the current HIP device, allocated
 *     and freed by the caller.  The library never allocates or frees device memory.  Pointer
 *     *lists* (peer_partials, out_slices, A_chunks) and `arrival_order` are HOST arrays that
 *     are read during the call only.
 *   - Streams are hipStream_t passed as void* (NULL = the default stream).  All calls are
 *     asynchronous: they validate, enqueue and return.  Nothing is enqueued when the
 *     returned status is not FLUX_OK.
 *   - Errors are returned as flux_status_t values; nothing throws or aborts.  A signal wait
 *     that exceeds `spin_timeout_ticks` is reported through flux_query_status after the
 *     stream has been synchronised (the kernel then leaves the affected tiles unwritten).
 *   - The status block keeps the first timeout until flux_init_buffers clears it.
 *   - Calls that share a workspace, an A_agg buffer or a signal array must not overlap in time.
 */
#ifndef FLUX_MI355_H_
#define FLUX_MI355_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLUX_MAX_RANKS 16
#define FLUX_MAX_M_TILES 1024      /* ceil(M / tile height) must not exceed this */
#define FLUX_MAX_N (1 << 21)       /* N must stay below this */

typedef enum {
  FLUX_OK = 0,
  FLUX_ERR_INVALID_ARG = 1,   /* null pointer, bad enum, misaligned base */
  FLUX_ERR_SHAPE = 2,         /* M % R != 0, N or K not a multiple of 8, sizes <= 0, a matrix of 2^31 elements or
                                 more, or N >= FLUX_MAX_N */
  FLUX_ERR_UNSUPPORTED = 3,   /* valid request the library has no kernel for */
  FLUX_ERR_WORKSPACE = 4,     /* workspace missing or smaller than flux_workspace_bytes */
  FLUX_ERR_HIP = 5,           /* a HIP runtime call failed (flux_last_hip_error has the code) */
  FLUX_ERR_TIMEOUT = 6        /* reported by flux_query_status only */
} flux_status_t;

typedef enum { FLUX_BF16 = 0, FLUX_F32 = 1 } flux_dtype_t;
typedef enum { FLUX_OP_RS = 0, FLUX_OP_AG = 1 } flux_op_t;

/* flux_problem_t.flags */
#define FLUX_FLAG_NO_SWIZZLE   0x1u  /* natural tile order: no rank shift / arrival alignment, no die remap */
#define FLUX_FLAG_NO_XCD_REMAP 0x2u  /* keep the visit order but do not regroup tiles per accelerator die */
#define FLUX_FLAG_COPY_MEMCPY  0x4u  /* AG copy driver = hipMemcpyAsync + stream write-value per
                                        communication tile instead of the copy kernel */

#define FLUX_FLAG_NO_TAIL_SPLIT 0x10u /* with split_k = 0: do not cut the tiles of a partly filled last
                                        round of the grid along K (see flux_split_plan) */

#define FLUX_FLAG_RS_WRITE_ONLY 0x20u /* flux_gemm_rs: Write branch of Alg. 1: no peers are read, each row of
                                        A.B is converted and stored into its owner's slice (the AlltoAll
                                        flavour of Sec. 3.1; flux_rs_reduce_slice is the reduction after it) */

#define FLUX_FLAG_RS_ATOMIC 0x80u     /* flux_gemm_rs: Reduce by atomic additions (Sec. 4.2, "Reduce", first form): no
                                        peers are read; each element of A.B is added, with one fp32 atomic
                                        addition, to its owner's slice, which holds what the other ranks have
                                        added so far (or zeros).  out_dtype must be FLUX_F32 (the paper, too,
                                        applies this form to selected data types only). */

#define FLUX_FLAG_AG_ABSENT_OWNERS 0x40u /* flux_ag_gemm without a copy kernel: share the pieces out over twice as
                                        many workgroups as the grid has, so that every second piece has an
                                        owner that never runs and is taken over by a workgroup that waits for
                                        it.  For tests of that take-over; costs time, never correctness. */

#define FLUX_FLAG_AG_COPY_UPFRONT 0x200u /* flux_ag_gemm without a copy kernel: move every remote chunk before the
                                        signal wait.  Without the flag a grid of several rounds moves only
                                        the chunks its first round needs up front and carries the others
                                        inside the first round's main loops (see flux_ag_deferred_tiles). */

#define FLUX_FLAG_NO_RESIDENT_GRID 0x100u /* flux_gemm_rs: always one workgroup per tile, dispatched by the hardware.
                                        Without the flag a grid of at least four rounds of 256x256 tiles with
                                        K <= 3072 runs as one resident workgroup per compute unit that walks
                                        the same block sequence (Sec. 4.1 order, in time), half of them half
                                        a tile period late, so that reduce epilogues (Sec. 4.2) and main
                                        loops of different units overlap.  Same results bit for bit. */

/* flux_gemm_ref_unfused phases */
#define FLUX_PHASE_GEMM 0x1
#define FLUX_PHASE_COMM 0x2

typedef struct flux_problem {
  int32_t M, N, K;          /* this rank's GEMM: A[M,K] . B[K,N]  (Alg. 1 / Alg. 2 operands)      */
  int32_t R, rank;          /* N_TP and rank_id                                                   */
  int32_t partial_dtype;    /* RS: dtype of the peer partials (flux_dtype_t); ignored for AG      */
  int32_t out_dtype;        /* dtype of out_slices / C (flux_dtype_t)                             */
  int32_t tile_config;      /* 0 = library picks; else an id from flux_tile_config_info           */
  int32_t split_k;          /* 0 = library picks; >1 cuts K over that many workgroups per tile    */
  uint32_t flags;           /* FLUX_FLAG_*                                                        */
  int32_t comm_tiles_per_chunk; /* AG: signals per chunk (Sec. 4.3 "communication tile size");
                                   0 or 1 = one per chunk; must divide M/R                        */
  int32_t copy_workgroups;  /* AG copy kernel grid size; 0 = library picks (for the fused call: no
                               copy kernel at all unless link_gbps is set, see flux_ag_gemm).  The
                               fused call uses at most 256: a communication tile moves in one
                               piece per workgroup.                                                */
  int32_t link_gbps;        /* AG transfer: 0 = at memory speed; else it stands for an inbound link
                               of that many GB/s: communication tile i of the transfer order is
                               not signalled before (i+1)*tile_bytes/link_gbps after the
                               transfer started (its data may move earlier)                      */
  int32_t reserved;         /* must be 0                                                          */
  uint64_t spin_timeout_ticks;  /* AG: bound on one signal wait, in 100 MHz wall-clock ticks;
                                   0 = library default (10 s).  The paper spins without bound.   */
  int64_t lda, ldb, ldc;    /* row pitches in elements, 0 = packed (K, N, N).  Multiples of 8, at
                               least a row long, below FLUX_MAX_N (ldc), the last element's index
                               below 2^31.
                               lda: A (flux_gemm_rs, the references) and the gathered matrix A_agg
                                    (flux_ag_gemm); the chunk sources A_chunks[r] are packed [M/R,K]
                                    (a local chunk handed over in place has A_agg's pitch).
                               ldb: B (rows of N values, or of K values with b_is_nk).
                               ldc: C, every out slice, and the staged slices that
                                    FLUX_FLAG_RS_WRITE_ONLY / flux_gemm_rs_notify write and
                                    flux_rs_reduce_slice / flux_rs_reduce_slice_ready read.
                               Peer partials are packed [M,N].  What lies between the end of a
                               row and the next row is neither read nor written.                  */
  int32_t b_is_nk;          /* 0: B is [K,N] (row k holds the N values B[k,:]).
                               1: B is [N,K], row n holding the K values B[:,n] -- the layout of a
                                  linear layer's weight, out features by in features; ldb is then the
                                  pitch of those rows (0 = K).  Same results bit for bit.          */
  int32_t reserved2;        /* must be 0                                                          */
} flux_problem_t;

/*
 * GEMM-ReduceScatter, fused (Alg. 1 with the Reduce branch).
 *   A, B            device, bf16, [M,K] and [K,N] ([N,K] with b_is_nk).
 *   peer_partials   (NULL allowed with FLUX_FLAG_RS_WRITE_ONLY / FLUX_FLAG_RS_ATOMIC) host array [R] of device pointers to [M,N] matrices of partial_dtype;
 *                   entry [rank] is ignored (may be NULL).
 *   out_slices      host array [R] of device pointers to [M/R,N] matrices of out_dtype, all
 *                   written (every element exactly once; with FLUX_FLAG_RS_ATOMIC: added to).
 *   workspace       device, >= flux_workspace_bytes(FLUX_OP_RS, p) bytes (may be NULL if 0),
 *                   initialised once with flux_init_buffers.
 */
int flux_gemm_rs(const flux_problem_t* p, const void* A, const void* B,
                 const void* const* peer_partials, void* const* out_slices,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * flux_gemm_rs for callers that cannot allocate or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments and results, but
 * what a call that cuts K needs beyond its inputs and outputs (arrival counters and parked fp32
 * partial tiles) lives in an array inside the library, FLUX_STATIC_SCRATCH_BYTES per GPU, held
 * from the time the library is loaded until the process ends.  The call allocates nothing.
 * A problem whose K cut needs more than that (flux_workspace_bytes says how much) is rejected with
 * FLUX_ERR_WORKSPACE before anything is enqueued; a problem that needs no workspace never touches
 * the array.  All calls on one GPU share that GPU's array, which keeps the last call's contents:
 * the call clears the counters itself (one small kernel ahead of the GEMM), and calls that overlap
 * in time on one GPU (different streams or threads) race.  Calls on one stream are safe.
 */
#define FLUX_STATIC_SCRATCH_BYTES (32u << 20)
int flux_gemm_rs_static(const flux_problem_t* p, const void* A, const void* B,
                        const void* const* peer_partials, void* const* out_slices, void* stream);

/*
 * AllGather-GEMM, fused (Alg. 2 kernel + the data transfer of Alg. 3, pull form).
 * Who moves the remote chunks (communication tile by communication tile in `arrival_order`,
 * setting each tile's signal when it is complete) depends on the problem:
 *   - link_gbps == 0, copy_workgroups == 0, no FLUX_FLAG_COPY_MEMCPY (the default): no copy kernel
 *     is launched and copy_stream stays unused.  The first workgroups of the GEMM grid (as many as
 *     run at once) share the pieces of the tiles out among themselves by index and move them
 *     before they look at their own signals; in a grid of several rounds they move only the chunks
 *     the first round reads that way and carry the others inside their main loops (see
 *     flux_ag_deferred_tiles, FLUX_FLAG_AG_COPY_UPFRONT).  A GEMM workgroup takes the whole
 *     register file of its compute unit, so a separate driver cannot run beside it: it would hold
 *     units the grid wants, and a waiting workgroup holds its unit anyway.
 *   - link_gbps > 0, copy_workgroups == 0, no FLUX_FLAG_COPY_MEMCPY: a transfer on a link's schedule,
 *     still without a copy kernel.  Workgroup w of the first round carries piece w of every remote
 *     tile: in batches while it waits for its own signals, two 16-byte vectors per thread and K slab
 *     inside its main loop, and it counts a tile in (the last piece sets the signal) no earlier
 *     than the link would have delivered it.  A driver that stands for a link would hold its
 *     compute units for as long as the transfer lasts, which no link does.  (Where the kernel
 *     cannot carry - tile configurations other than 256x256 two-stage, ragged shapes, more than 32
 *     remote tiles - this falls back to the paced copy kernel below.)  The same holds for stream
 *     capture as for the default form.
 *   - copy_workgroups > 0 (or link_gbps > 0 where the grid cannot carry): the driver of Alg. 3 is a
 *     kernel on copy_stream, paced if link_gbps > 0.  A
 *     GEMM workgroup that has to wait for a tile moves pieces of that tile which no one has started
 *     on (pieces are claimed, so nothing is moved twice); the call therefore also completes when
 *     the GEMM grid takes every compute unit before the driver got one.  A paced driver
 *     (link_gbps > 0) stands for a link, so workgroups only step in while part of the driver has
 *     not started.
 *   - FLUX_FLAG_COPY_MEMCPY: the driver is hipMemcpyAsync plus a stream write per tile and the
 *     GEMM only waits.
 * In the first two cases a piece is claimed before it is moved, whoever moves it, and a workgroup
 * that waits takes over unclaimed pieces of the tiles it waits for, so a mover that has not been
 * given a compute unit yet cannot stall the grid.
 * Stream capture: in the default form the call is kernel launches on compute_stream only (one, or
 * two if the local chunk has to be copied into place) and everything that changes from call to
 * call lives in the workspace, so it may be recorded in a HIP graph and replayed.  The forms with a
 * driver take a fresh claim id from the host on every call: under stream capture they return
 * FLUX_ERR_UNSUPPORTED.
 *   A_chunks        host array [R] of device pointers, chunk r = [M/R,K] bf16 ("A_list").
 *   A_agg           device [M,K] bf16 (row pitch lda), written by the call.  If A_chunks[rank] already points
 *                   at A_agg + rank*(M/R)*lda the local chunk is not copied.  16-byte alignment is
 *                   required; with 128-byte alignment and a row pitch that is a multiple of 64 no cache line holds
 *                   rows of two communication tiles, and a workgroup leaves its signal wait without
 *                   invalidating its die's L2 (one to two microseconds per workgroup otherwise).
 *   B, C            device, [K,N] bf16 ([N,K] with b_is_nk) and [M,N] out_dtype.
 *   signals         device uint32[R * comm_tiles_per_chunk] ("signal_list").  Must be in the preset
 *                   state on entry (local communication tiles 1, the others 0): preset once
 *                   with flux_init_buffers, as the paper presets at operator initialisation;
 *                   a call that completes without timeout leaves them preset again (the reset
 *                   after the GEMM of Sec. 4.3 "Signals", done by the last workgroup that has
 *                   passed its wait).  After a timeout call flux_init_buffers again.
 *   arrival_order   host int32[R-1]: the remote ranks in the order the copy driver transfers
 *                   them; NULL = ring order starting after `rank` (Sec. 4.3).
 *   workspace       device, >= flux_workspace_bytes(FLUX_OP_AG, p), initialised once with
 *                   flux_init_buffers (status block, counters, piece claims).
 *   compute_stream  the GEMM kernel's stream; on return of the call it is ordered after the
 *                   GEMM, the copy driver and the signal reset.
 *   copy_stream     the copy driver's stream; must differ from compute_stream.
 *                   HIP maps streams onto a few hardware queues (GPU_MAX_HW_QUEUES, 4 by default)
 *                   and a queue hands out its packets in order: if both streams land on one queue
 *                   the driver and the GEMM run one after the other, correctly but without overlap.
 *                   Successively created streams go to different queues.
 */
int flux_ag_gemm(const flux_problem_t* p, const void* const* A_chunks, void* A_agg,
                 const void* B, void* C, uint32_t* signals, const int32_t* arrival_order,
                 void* workspace, size_t workspace_bytes,
                 void* compute_stream, void* copy_stream);

/*
 * Non-overlapped baseline (Sec. 2.3: the reference point of Eq. 2), everything on one stream.
 *   op = FLUX_OP_RS:  FLUX_PHASE_GEMM  C = A.B (C: device [M,N] of out_dtype, a temporary);
 *                     FLUX_PHASE_COMM  out_slices[r] = C + sum peers (separate kernel).
 *   op = FLUX_OP_AG:  FLUX_PHASE_COMM  copy all chunks into A_agg (no signals);
 *                     FLUX_PHASE_GEMM  C = A_agg.B.
 *   `phases` selects which of the two to enqueue (both: communication and GEMM in dependency
 *   order).  Arguments not used by `op` may be NULL; `workspace` as for the fused call when
 *   flux_workspace_bytes is non-zero for the problem (FLUX_OP_RS: only when K is split).  The GEMM kernel is the same tile
 *   configuration the fused call would use, without prologue wait or reduce epilogue.
 */
int flux_gemm_ref_unfused(int op, int phases, const flux_problem_t* p,
                          const void* A, const void* const* A_chunks, void* A_agg,
                          const void* B, const void* const* peer_partials,
                          void* const* out_slices, void* C,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of device workspace the given problem needs (0 on invalid problems). */
size_t flux_workspace_bytes(int op, const flux_problem_t* p);

/*
 * One-time initialisation of caller-owned buffers (the paper's operator-initialisation step,
 * Sec. 4.3 "Signals"): clears the workspace header (arrival counters, status block) and, for
 * FLUX_OP_AG, presets `signals` (local communication tiles 1, the others 0).  `workspace` or
 * `signals` may be NULL to skip that part.  Enqueued on `stream`.
 */
int flux_init_buffers(int op, const flux_problem_t* p, void* workspace, size_t workspace_bytes,
                      uint32_t* signals, void* stream);

/*
 * Reads the status block a finished flux_ag_gemm left in `workspace` (blocking device-to-host
 * copy; synchronise the streams first).  code = FLUX_OK or FLUX_ERR_TIMEOUT, detail = index
 * of the first signal that timed out.
 */
int flux_query_status(const void* workspace, int32_t* code, int32_t* detail);

/*
 * TileCoord of Alg. 1 / Alg. 2 as the kernels compute it (host function, for tests):
 * linear workgroup id -> (m_tile, n_tile) for the tile configuration the call would use.
 */
int flux_tile_coord(int op, const flux_problem_t* p, const int32_t* arrival_order,
                    int32_t block, int32_t* m_tile, int32_t* n_tile);

/*
 * The local reduction that follows the AlltoAll when flux_gemm_rs runs with FLUX_FLAG_RS_WRITE_ONLY
 * (Sec. 3.1: ReduceScatter = AlltoAll + reduction; Sec. 4.2): `staged` is a host array [R] of device
 * pointers, staged[j] = the [M/R,N] partial (partial_dtype) that rank j wrote for THIS rank's slice;
 * out [M/R,N] (out_dtype) = their sum in rank order, fp32, converted once.  One kernel on `stream`.
 */
int flux_rs_reduce_slice(const flux_problem_t* p, const void* const* staged, void* out, void* stream);

/*
 * Reduce with tile-ready counters (Sec. 4.2, "Reduce", second form: the producers write their tiles
 * to the destination and raise a flag per tile; a reducer on the destination takes the tiles as
 * they come up).  Every rank's GEMM scatters its product by owner (the Write branch of Alg. 1) and
 * counts each tile in; the owner's reducer waits tile by tile and sums the staged partials.
 *
 * flux_gemm_rs_notify   producer: flux_gemm_rs with FLUX_FLAG_RS_WRITE_ONLY (implied) whose stores go
 *                       through to memory and whose workgroups, after their tile's last store is
 *                       acknowledged, add one to tile_ready[m_tile * tiles_n + n_tile] (the tile grid of
 *                       the whole [M,N] product under the call's tile configuration; flux_rs_ready_count
 *                       entries).  A tile cut along K is counted once, by the workgroup that writes it.
 * flux_rs_reduce_slice_ready
 *                       consumer for the slice of rank p->rank: `staged` as for flux_rs_reduce_slice; for
 *                       every tile that overlaps the slice it waits until the counter has reached
 *                       `producers` (bounded by p->spin_timeout_ticks like a signal wait: a tile that
 *                       times out is left unwritten and reported through flux_query_status on `workspace`,
 *                       detail = index of the counter), then writes out = sum of the staged rows in rank
 *                       order, fp32, converted once.  It must be given the same M, N, K, R and tile_config
 *                       as the producers (the counters are per producer tile).  `workspace`: device,
 *                       at least 32 KiB, cleared once with flux_init_buffers(FLUX_OP_RS, ...).
 * tile_ready            device uint32[flux_rs_ready_count(p)], zero before the first producer starts;
 *                       neither side resets it (on one GPU the counters of a tile that spans several
 *                       slices are shared by their owners): clear it between rounds.
 * The consumer may be enqueued before, beside or after the producers; enqueue it on a stream of its own
 * AFTER the producers so that it can never sit ahead of one of them in a hardware queue.
 */
int flux_gemm_rs_notify(const flux_problem_t* p, const void* A, const void* B, void* const* out_slices,
                        uint32_t* tile_ready, void* workspace, size_t workspace_bytes, void* stream);
int flux_rs_reduce_slice_ready(const flux_problem_t* p, const void* const* staged, void* out,
                               uint32_t* tile_ready, int32_t producers,
                               void* workspace, size_t workspace_bytes, void* stream);
int32_t flux_rs_ready_count(const flux_problem_t* p);

/*
 * Medium-grained baseline: the decomposition the paper compares against (Sec. 2.2): the GEMM is
 * cut into R GEMMs of M/R rows, one per slice / chunk, and the communication of one part runs on
 * comm_stream beside the GEMM of the next on compute_stream.
 *   op = FLUX_OP_RS:  for each slice (ring order after `rank`, own slice last): C rows = A rows . B
 *                     on compute_stream, then out_slices[slice] = C rows + sum peers on comm_stream.
 *   op = FLUX_OP_AG:  chunk copies into A_agg on comm_stream in `arrival_order`; the GEMM of a
 *                     chunk's rows on compute_stream as soon as that chunk has been copied (local
 *                     chunk first).
 * Arguments as for flux_gemm_ref_unfused (C: device [M,N] of out_dtype; for RS a temporary).  Each
 * part is planned like a GEMM of its own shape; if that plan cuts K, `workspace` must hold
 * flux_chunked_workspace_bytes(op, p) bytes, initialised with flux_init_buffers.  The two streams
 * must differ; on return compute_stream is ordered after everything the call enqueued.
 */
int flux_gemm_ref_chunked(int op, const flux_problem_t* p,
                          const void* A, const void* const* A_chunks, void* A_agg, const void* B,
                          const void* const* peer_partials, void* const* out_slices, void* C,
                          const int32_t* arrival_order, void* workspace, size_t workspace_bytes,
                          void* compute_stream, void* comm_stream);
size_t flux_chunked_workspace_bytes(int op, const flux_problem_t* p);

/*
 * Tuner (Sec. 4.4; the communication tile size of Sec. 4.3 among the knobs).  Times the fused call
 * on the caller's own buffers for every tile configuration that accepts the shape, for few-row
 * shapes (M <= 256) also with half and twice the library's number of K parts, and, for the
 * AllGather, for communication tiles of the chunk height halved down to the GEMM tile height (at
 * most 8 per chunk), and with the other form of prologue or epilogue where the library would pick
 * one by rule (FLUX_FLAG_AG_COPY_UPFRONT, FLUX_FLAG_NO_RESIDENT_GRID), against what the library picks
 * by itself, and writes the fastest problem description to *tuned (a copy of *p with tile_config,
 * split_k, comm_tiles_per_chunk and such a flag filled in; the library's own pick wins unless a
 * candidate is more than 2 % faster).  *ms_best / *ms_default
 * (either may be NULL) receive the median time per call of the winner and of the library's pick.
 * Buffers as for flux_gemm_rs / flux_ag_gemm; outputs are overwritten with the (same) result.  The
 * workspace must hold flux_autotune_workspace_bytes(op, p) bytes (candidates that need more than
 * workspace_bytes are skipped) and `signals` flux_autotune_signal_count(p) words (signal_count says
 * how many there are).  `reps` timed samples per candidate (0 = 5).  The call blocks until done and
 * leaves workspace and signals initialised for *tuned.  Not for use under stream capture.
 */
int flux_autotune_rs(const flux_problem_t* p, const void* A, const void* B,
                     const void* const* peer_partials, void* const* out_slices,
                     void* workspace, size_t workspace_bytes, void* stream, int32_t reps,
                     flux_problem_t* tuned, float* ms_best, float* ms_default);
int flux_autotune_ag(const flux_problem_t* p, const void* const* A_chunks, void* A_agg, const void* B, void* C,
                     uint32_t* signals, int32_t signal_count, const int32_t* arrival_order,
                     void* workspace, size_t workspace_bytes, void* compute_stream, void* copy_stream,
                     int32_t reps, flux_problem_t* tuned, float* ms_best, float* ms_default);
size_t flux_autotune_workspace_bytes(int op, const flux_problem_t* p);
int flux_autotune_signal_count(const flux_problem_t* p);

/*
 * How a call would cut K: the first *full_tiles tiles in TileCoord order are computed by one
 * workgroup each, the remaining *split_tiles tiles by *split_k workgroups each (a uniform split has
 * full_tiles = 0; no split has split_k = 1 and split_tiles = all tiles).  The grid has
 * full_tiles + split_tiles * split_k workgroups.  Host function; any pointer may be NULL.
 */
int flux_split_plan(int op, const flux_problem_t* p, int32_t* full_tiles, int32_t* split_tiles,
                    int32_t* split_k);

/*
 * Whether flux_gemm_rs would run this problem as a grid of resident workgroups (see
 * FLUX_FLAG_NO_RESIDENT_GRID): returns the number of resident workgroups (0: one workgroup per block of
 * flux_split_plan, dispatched by the hardware) and, in *delay_ticks, how late every second group of
 * eight of them starts (100 MHz ticks).  The blocks and their order (flux_tile_coord, flux_split_plan)
 * and the tile trace (one record per block) are the same in both forms.  Host function.
 */
int32_t flux_rs_resident_grid(const flux_problem_t* p, uint32_t* delay_ticks);

/*
 * How many of the (R-1) * comm_tiles_per_chunk remote communication tiles flux_ag_gemm (forms without a
 * copy kernel) has its first round of workgroups carry themselves instead of moving them before the
 * signal wait (Sec. 3.2: tiles whose data has arrived compute while the rest is on its way): the last
 * that many tiles of the transfer order; all of them when link_gbps > 0.  0: everything is moved up
 * front, or a copy kernel moves it.  Host function.
 */
int32_t flux_ag_deferred_tiles(const flux_problem_t* p);

/* Tile configuration a call would use: tile sizes, K split and die count used for the remap. */
int flux_tile_shape(int op, const flux_problem_t* p, int32_t* tile_m, int32_t* tile_n,
                    int32_t* tile_k, int32_t* split_k, int32_t* n_xcd);

/* Enumerates tile configurations: returns FLUX_OK and fills the sizes for ids 1..count. */
int flux_tile_config_count(void);
int flux_tile_config_info(int32_t id, int32_t* tile_m, int32_t* tile_n, int32_t* tile_k);

/* Communication order of Sec. 4.3 (ring starting after the local rank): fills order[R-1]. */
int flux_default_order(int32_t rank, int32_t R, int32_t* order);

/*
 * Measurement hook: the next flux_gemm_rs / flux_ag_gemm / flux_gemm_ref_unfused call made by
 * this thread records `start` immediately before and `stop` immediately after its GEMM kernel
 * launch, on the stream that kernel runs on (hipEvent_t handles passed as void*; the pair is
 * consumed by that call).  Passing NULLs cancels a pending pair.  The elapsed time between
 * the two is the kernel's duration including any in-kernel signal waits.
 */
int flux_profile_next_gemm(void* start_event, void* stop_event);

/*
 * Tile trace (Sec. 4.1: which workgroup computes which tile, and in what order they are dispatched;
 * Sec. 3.2: how long a tile waits for its signals).  The next flux_gemm_rs / flux_ag_gemm /
 * flux_gemm_ref_unfused call made by this thread has every workgroup of its GEMM kernel write one
 * record, indexed by workgroup id, into `records` (device memory, 16-byte aligned, at least
 * 64 bytes times the grid size full_tiles + split_tiles * split_k of flux_split_plan; a call whose
 * grid does not fit returns FLUX_ERR_WORKSPACE and enqueues nothing).  The request is consumed by
 * that call; NULL cancels a pending one.  Clocks are the GPU's 100 MHz wall clock, comparable
 * between workgroups of one launch.  Tracing costs a few stores per workgroup and makes the last
 * stamp wait for the workgroup's stores; results are unchanged.
 */
typedef struct flux_trace_record {
  uint32_t block;       /* workgroup id                                                          */
  uint32_t m_tile;      /* TileCoord of Alg. 1 / Alg. 2 as the kernel computed it                */
  uint32_t n_tile;
  uint32_t k_part;      /* bits [15:0]: index of the K part; bit 16: the tile is cut along K     */
  uint32_t die;         /* accelerator die (XCC) the workgroup ran on                            */
  uint32_t hw_id;       /* raw hardware id register: wave [3:0], SIMD [5:4], CU [11:8], shader
                           array [12], shader engine [15:13]                                     */
  uint32_t tile;        /* index of the tile in TileCoord order                                  */
  uint32_t reserved;
  uint64_t t_start;     /* kernel entry                                                          */
  uint64_t t_ready;     /* past the signal wait (AllGather; equals t_start otherwise)            */
  uint64_t t_main_end;  /* main loop done                                                        */
  uint64_t t_end;       /* epilogue (or K-part hand-over) done, stores acknowledged              */
} flux_trace_record_t;
int flux_trace_next_call(void* records, size_t bytes);

const char* flux_status_string(int status);
int flux_last_hip_error(void);       /* hipError_t of the most recent FLUX_ERR_HIP on this thread */
int flux_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLUX_MI355_H_ */
