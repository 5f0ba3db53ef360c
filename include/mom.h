/*
 * libmom — C ABI of the MI355X (gfx950) prefill hot path of MOM
 * ("Memory-efficient Offloaded Mini-sequence Inference", arXiv 2504.12526).
 *
 * Conventions for every call
 *   - bf16 tensors are arrays of 16-bit patterns (upper half of IEEE binary32),
 *     row-major, densely packed.
 *   - Unless a parameter says "host", pointers are DEVICE pointers on the
 *     current HIP device.  The caller owns every buffer, stream and event.
 *   - `stream` parameters are `hipStream_t` passed as `void*` (NULL = the
 *     default stream).  Calls only ENQUEUE work; they never synchronise.
 *     Results are valid once the caller has synchronised the stream (or the
 *     event the call records).
 *   - The library allocates nothing.  The only state it keeps is what it looks up once per
 *     device (compute-unit count, address of the static workspace of
 *     mom_mlp_prefill_static) and the testing overrides at the end of this header.
 *   - Return value: a `mom_status`; 0 is success.  Arguments are validated
 *     before anything is enqueued, so a non-zero status other than
 *     MOM_ERR_HIP means nothing was launched.
 *
 * Weight layout (the paper states only the mathematical shapes d->I, I->d):
 * every weight is stored "output features x input features", so each
 * contraction runs over the contiguous axis of both operands:
 *   W_gate [I,H]   W_up [I,H]   W_down [H,I]   W_lm [V,H]
 */
#ifndef MOM_H
#define MOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOM_OK = 0,
    MOM_ERR_NULL = 1,      /* a required pointer is NULL */
    MOM_ERR_SHAPE = 2,     /* negative / zero / unsupported extent (H, I must be multiples of 32) */
    MOM_ERR_ALIGN = 3,     /* a pointer is not 16-byte aligned */
    MOM_ERR_ALIAS = 4,     /* an output or the workspace overlaps an input */
    MOM_ERR_WORKSPACE = 5, /* workspace_bytes is smaller than mom_mlp_workspace_bytes() */
    MOM_ERR_HIP = 6,       /* the HIP runtime reported an error while enqueueing */
    MOM_ERR_HOST = 7       /* a host buffer is not page-locked memory known to the HIP runtime */
} mom_status;

/* Human-readable, static string for a status value. */
const char *mom_status_string(int status);

/*
 * Optional set-up for the current HIP device: looks up what the other calls otherwise look up
 * on their first use on a device (the compute-unit count, the device address of the static
 * workspace of mom_mlp_prefill_static), so that those calls make no runtime query afterwards.
 * Call it once per device, with that device current, e.g. before a stream capture.  Returns
 * MOM_ERR_HIP when there is no usable device.
 */
int mom_init(void);

/*
 * Bytes of workspace mom_mlp_prefill needs: C*I*2 with C = mini_seq if
 * 0 < mini_seq < S, else S.  This is the mini-sequence intermediate of the
 * paper's Eq. 3 (one C x I bf16 tensor), against S*I*2 for the full-sequence
 * evaluation of Eq. 1.  Returns 0 for S <= 0 or invalid H / I / mini_seq.
 */
size_t mom_mlp_workspace_bytes(int64_t S, int64_t H, int64_t I, int64_t mini_seq);

/*
 * Mini-sequence SwiGLU MLP (Algorithm 1, else-branch; Section 3.3 "Llama MLP
 * Layer"):
 *     out = ( silu(x W_gate^T) .* (x W_up^T) ) W_down^T
 * evaluated over ceil(S/C) mini-sequences of C = mini_seq rows (the last one
 * shorter when C does not divide S); each mini-sequence's C x I intermediate is
 * written to `workspace` and consumed before the next one overwrites it, and its
 * output rows land directly at their place in `out` (the concat).
 *
 *   x        [S,H] bf16      in
 *   W_gate   [I,H] bf16      in
 *   W_up     [I,H] bf16      in
 *   W_down   [H,I] bf16      in
 *   out      [S,H] bf16      out
 *   workspace  at least mom_mlp_workspace_bytes(S,H,I,mini_seq) bytes, scratch
 *   mini_seq   rows per mini-sequence; 0 or >= S evaluates the whole sequence
 *              at once through the same kernels (workspace S*I*2 bytes)
 *
 * Arithmetic: bf16 operands, fp32 accumulation on the matrix cores, SiLU and
 * the gate*up product in fp32, one round-to-nearest-even to bf16 into the
 * workspace, fp32 accumulation of the down projection, one rounding to bf16.
 * Every output row is computed by an instruction sequence that does not depend
 * on mini_seq or on the row's position, so any two values of mini_seq give
 * bit-identical `out`.
 *
 * S = 0 is a no-op returning MOM_OK.  H and I must be positive multiples of 32.
 * All work is enqueued on `stream` in order (2 kernels per mini-sequence).
 * The kernels exist in several tile forms with bit-identical results; the library picks one per
 * launch (mom_debug_force_gemm_form overrides the choice, for tests).
 */
int mom_mlp_prefill(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                    int64_t S, int64_t H, int64_t I, int64_t mini_seq,
                    void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * mom_mlp_prefill for callers that cannot provide (or allocate) a workspace: code under HIP graph
 * capture, tight serving loops, harnesses in which nothing may call hipMalloc.  Same computation,
 * same kernels and same bits as mom_mlp_prefill; the mini-sequence intermediate lives in a
 * MOM_STATIC_WORKSPACE_BYTES array that is part of the library's device image (each device the
 * library is used on holds its copy until the process ends).  The call allocates nothing and
 * frees nothing.
 *   Limit: min(mini_seq, S) * I * 2 <= MOM_STATIC_WORKSPACE_BYTES (e.g. 2048 rows at I = 14336),
 *   else MOM_ERR_WORKSPACE and nothing is enqueued.  Other arguments and errors as mom_mlp_prefill.
 *   The device address of the array is looked up on the first call on a device (or by mom_init,
 *   which callers under stream capture should call beforehand).
 *   All calls on one device share the one array: every element a call reads it has written
 *   before, so nothing needs clearing between calls, but two calls that may run concurrently on
 *   one device (different streams without an ordering between them) race.
 */
#define MOM_STATIC_WORKSPACE_BYTES (64u << 20)
int mom_mlp_prefill_static(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                           int64_t S, int64_t H, int64_t I, int64_t mini_seq, void *out, void *stream);

/*
 * The same computation and the same bits as mom_mlp_prefill, scheduled on two streams with a
 * double-buffered workspace (2 * C * I * 2 bytes: still O(C*I), the bound of the paper's Eq. 3):
 * the down projection of mini-sequence c runs on `stream2` beside the gate/up projection of
 * mini-sequence c+1 on `stream`, so the CUs that the last, partly filled round of tiles of one
 * kernel leaves idle work on the other.  Pays off when a mini-sequence has few tiles (mini_seq
 * of 2048 rows and below on a 256-CU device); with many it equals mom_mlp_prefill.
 *   workspace        at least mom_mlp_pipelined_workspace_bytes(S,H,I,mini_seq) bytes
 *   stream, stream2  two streams of the current device (stream2 should differ from stream).  The
 *                    call orders stream2 after the work already enqueued on stream, and stream
 *                    after the last kernel on stream2: the caller synchronises `stream` only.
 *   events           host array of n_events >= 5 hipEvent_t created by the caller (disable-timing
 *                    events are fine); the first five are re-recorded freely during the call.
 *                    Fewer than five: MOM_ERR_SHAPE
 * With a single mini-sequence (mini_seq 0 or >= S), or where the schedule was measured not to pay
 * (a down projection that fills more than half of the CUs by itself, or mini-sequences so short
 * that both projections are latency-bound), this is mom_mlp_prefill on `stream`
 * (mom_debug_force_pipeline forces the two-stream schedule, for tests).
 */
size_t mom_mlp_pipelined_workspace_bytes(int64_t S, int64_t H, int64_t I, int64_t mini_seq);
int mom_mlp_prefill_pipelined(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                              int64_t S, int64_t H, int64_t I, int64_t mini_seq,
                              void *out, void *workspace, size_t workspace_bytes,
                              void *stream, void *stream2, void **events, int64_t n_events);

/*
 * The same computation with a HIP event recorded on `stream` before the first
 * kernel and after every kernel: events[0], then for mini-sequence c the event
 * events[1+2c] after its gate/up kernel and events[2+2c] after its down kernel.
 * `events` is a host array of n_events `hipEvent_t` created by the caller;
 * n_events must be at least 1 + 2*ceil(S/C).  For per-kernel timing only.
 */
int mom_mlp_prefill_events(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                           int64_t S, int64_t H, int64_t I, int64_t mini_seq,
                           void *out, void *workspace, size_t workspace_bytes, void *stream,
                           void **events, int64_t n_events);

/*
 * Last-token LM head (Algorithm 1, if-branch; Section 3.3: one projected token
 * needs V outputs, not S*V):
 *     logits[v] = sum_k x_last[k] * W_lm[v,k]
 *   x_last [H] bf16 in,  W_lm [V,H] bf16 in,  logits [V] fp32 out.
 * fp32 accumulation, fp32 result (no rounding before an argmax / softmax).
 * H must be a positive multiple of 32 and at most 32768; V = 0 is a no-op.
 */
int mom_lmhead_last(const void *x_last, const void *W_lm, int64_t V, float *logits,
                    int64_t H, void *stream);

/*
 * Last-token MLP (Algorithm 1, if-branch: O_last = MLP(A_last)), tuned for one token: two
 * bandwidth-bound matrix-vector passes that stream each weight exactly once,
 *     h = silu(x_last W_gate^T) .* (x_last W_up^T)   [I] bf16 -> workspace
 *     out_last = h W_down^T                          [H] bf16
 *   x_last [H] bf16 in; W_gate, W_up [I,H], W_down [H,I] bf16 in; out_last [H] bf16 out;
 *   workspace: at least I*2 bytes of scratch.
 * Same arithmetic contract as mom_mlp_prefill (fp32 accumulation, fp32 SiLU and product, one
 * rounding to bf16 per projection), but the summation order differs from the matrix-core path, so
 * the result agrees with mom_mlp_prefill(S=1) to rounding, not bit for bit.
 * H and I must be positive multiples of 32 and at most 32768.
 */
int mom_mlp_last(const void *x_last, const void *W_gate, const void *W_up, const void *W_down,
                 int64_t H, int64_t I, void *out_last, void *workspace, size_t workspace_bytes,
                 void *stream);

/*
 * KV-cache offload of one layer (Algorithm 1 "offload"; Section 3.2): byte-exact
 * asynchronous copy of k then v (bytes_each bytes each, device) to
 * `pinned_host` (host, page-locked, at least 2*bytes_each bytes; k at offset 0,
 * v at offset bytes_each) on `stream`, meant to be a side stream so the copy
 * runs under the MLP kernels.  Pageable host memory is refused with MOM_ERR_HOST before
 * anything is enqueued: the runtime would stage such a copy and block the caller.
 *   order_event      hipEvent_t; if not NULL it is recorded on producer_stream first and `stream`
 *                    waits for it, so the copy starts after the work that produced k and v
 *   producer_stream  the stream that produced k and v; NULL means the default stream (which does
 *                    NOT order itself against a non-blocking side stream, so pass order_event
 *                    in that case too).  Ignored when order_event is NULL; passing a non-NULL
 *                    producer_stream without an order_event is an error (MOM_ERR_NULL)
 *   done_event       if not NULL, recorded on `stream` after both copies; the
 *                    device k/v may be reused once it has completed
 * bytes_each = 0 is a no-op (events are still recorded).
 */
int mom_kv_offload(const void *k, const void *v, void *pinned_host, void *stream,
                   size_t bytes_each, void *producer_stream, void *order_event,
                   void *done_event);

/*
 * KV-cache reload before decode (Algorithm 1, if-branch: "transfer offloaded cache back to GPU";
 * Section 3.2): the mirror of mom_kv_offload.  Asynchronous copy of bytes_each bytes from
 * `pinned_host` (host, page-locked; k at offset 0, v at offset bytes_each) into device k and v
 * on `stream`; `done_event`, if not NULL, is recorded after both copies.  Pageable host memory
 * is refused with MOM_ERR_HOST.  Ordering is the caller's: make `stream` wait for the last work that still reads the old contents of k and v
 * before this call, and make the consumers of k and v wait for `done_event`.
 */
int mom_kv_reload(const void *pinned_host, void *k, void *v, void *stream, size_t bytes_each,
                  void *done_event);

/*
 * Testing aids (they follow no passage of the paper; process-wide, not meant for production).
 *
 * mom_debug_force_gemm_form: every later matrix-core launch uses tiles of tile_edge x tile_edge
 * (256, 128 or 64) and an LDS ring of ring_slots slots (256: 5; 128: 5 or 10; 64: 5, 10 or 20;
 * 0 = the library's choice for that edge) whatever the launch's size.  tile_width (only with
 * tile_edge 256; 0 = 256) is the number of weight rows a tile stages: 256, 224, 192, 160 or 128
 * make the tiles of the down projection 256 token rows x tile_width output columns; 192 also makes
 * the gate/up tiles 256 token rows x 96 output columns (96 rows of W_gate and 96 of W_up) instead
 * of 128.  (0, 0, 0) gives the choice back to the library.
 * All forms give identical bits.  Other values: MOM_ERR_SHAPE, nothing changes.
 *
 * mom_debug_force_pipeline: on != 0 makes mom_mlp_prefill_pipelined use its two-stream schedule
 * whenever there is more than one mini-sequence, also where it was measured not to pay.
 */
int mom_debug_force_gemm_form(int tile_edge, int ring_slots, int tile_width);
int mom_debug_force_pipeline(int on);

/*
 * Measurement aid: the rate the matrix cores of this machine sustain on given operand values.
 * Launches `workgroups` workgroups of 4 wavefronts (one per SIMD); every wavefront fills 16 + 16
 * operand fragments once from a_bf16 / b_bf16 (device, bf16, a_bytes / b_bytes >= 16 and
 * multiples of 16 are used; indices wrap) and then runs `iters` times 128
 * v_mfma_f32_16x16x32_bf16 on 64 accumulator blocks in registers, with no LDS and no memory
 * traffic.  order 0: two in a row on each block (the two K-halves of a stage), the order of the
 * matrix-core kernels; order 1: the first of each pair on all 64 blocks, then the second (what the
 * kernels did before: the difference is what accumulating back to back saves).  Other values:
 * MOM_ERR_SHAPE.
 *   flop of a launch = workgroups * 4 * iters * 128 * 16384
 *   sink   device, at least workgroups * 256 floats; receives one checksum per lane
 * Timed by the caller with events on `stream`.  The power an MFMA draws depends on the values
 * it multiplies, and the chip sets its clock by its power limit, so the rate measured here on a
 * workload's own tensors is the ceiling of any kernel built from this instruction on that data,
 * as opposed to the datasheet peak at the maximum clock.
 */
int mom_debug_mfma_probe(const void *a_bf16, size_t a_bytes, const void *b_bf16, size_t b_bytes,
                         int64_t iters, int workgroups, int order, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOM_H */
