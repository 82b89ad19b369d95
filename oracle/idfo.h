/*
 * CPU oracle for the incremental depth-first CNN update (Binas & Bengio,
 * "Low-memory convolutional neural networks through incremental depth-first
 * processing").
 *
 * TEST INFRASTRUCTURE ONLY.  This library is the slow, plain reference the GPU
 * library is checked against and the CPU baseline that is timed beside it.  It
 * shares no code with the GPU library and must never be called from it.
 *
 * Two families, each in a floating-point (double) and an integer (int64_t)
 * flavour:
 *
 *   idfo_dense_*   -- the conventional layer-by-layer network of the paper's
 *                     first equation in Sec. 3 (h = f(sum w h + b)), evaluated
 *                     one whole layer after the other (Fig. 1 a-c).
 *   idfo_stream_*  -- the paper's scheme (Sec. 3, the stateful neuron, the event
 *                     definition and the event-delivery rule): every non-zero
 *                     value of an arriving row is one event, delivered one at a
 *                     time into the stateful pre-activations c of the next
 *                     layer; a row of c that no future input can change is
 *                     activated, emitted depth-first to the next layer and
 *                     forgotten (Fig. 2).  Only a rolling set of K_h rows per
 *                     layer is ever held.
 *
 * Layouts (all row-major, channel last):
 *   input / activations   [rows][W][C]
 *   conv weights          [C_out][C_in][K_h][K_w]
 *   bias                  [C_out] or NULL (= zero, the paper's WLOG assumption)
 * 1-D signals are W = 1, K_w = 1; the streaming axis is "rows".
 */
#ifndef IDFO_H
#define IDFO_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { IDFO_CONV = 0, IDFO_MAXPOOL = 1 };
enum { IDFO_ACT_NONE = 0, IDFO_ACT_RELU = 1, IDFO_ACT_RELU_SHR_CLAMP = 2 };
enum { IDFO_ROUND_NONE = 0, IDFO_ROUND_BF16 = 1 };

typedef struct {
    int kind;            /* IDFO_CONV or IDFO_MAXPOOL (2x2, stride 2, no padding) */
    int c_in, c_out;     /* pool: c_out == c_in                                    */
    int k_h, k_w;        /* pool: 2, 2 (1-D pool: 2, 1)                            */
    int s_h, s_w;
    int p_h, p_w;        /* zero padding on top/left (and bottom/right)            */
    int act;             /* IDFO_ACT_*                                             */
    int shr, clamp_hi;   /* for IDFO_ACT_RELU_SHR_CLAMP: min(clamp_hi, max(c,0)>>shr) */
} idfo_layer;

/* Output height/width of one layer for an input of that height/width
 * (floor((n + 2p - k)/s) + 1; 0 when the kernel does not fit). */
int idfo_out_size(int n_in, int k, int s, int p);

/* bf16 round-to-nearest-even of a double (returned as the exactly representable
 * double).  Used for the emulated rounding of emitted activations. */
double idfo_round_bf16(double v);

/* ---- dense, layer by layer ------------------------------------------------
 * x:   [H][W][C0]
 * w/b: one pointer per layer (entries for pool layers ignored, may be NULL)
 * emit_round: rounding applied to every conv layer's activation except the
 *             last layer's (float flavour only)
 * layer_out:  NULL, or n_layers pointers (each NULL or a buffer large enough
 *             for that layer's [H_o][W_o][C_out] activations)
 * out: the last layer's activations.
 * Returns 0, or -1 on an inconsistent description. */
int idfo_dense_f64(const idfo_layer *layers, int n_layers, int H, int W, int C0,
                   const double *x, const double *const *w, const double *const *b,
                   int emit_round, double *out, double *const *layer_out);
int idfo_dense_i64(const idfo_layer *layers, int n_layers, int H, int W, int C0,
                   const int64_t *x, const int64_t *const *w, const int64_t *const *b,
                   int emit_round, int64_t *out, int64_t *const *layer_out);

/* ---- streaming, event by event ---------------------------------------------
 * H = 0 means an unbounded 1-D style stream (only zero top/bottom padding is
 * then allowed).  With H > 0 the stream re-arms itself after row H-1. */
typedef struct idfo_stream_f64 idfo_stream_f64;
typedef struct idfo_stream_i64 idfo_stream_i64;

idfo_stream_f64 *idfo_stream_new_f64(const idfo_layer *layers, int n_layers, int H, int W, int C0,
                                     const double *const *w, const double *const *b,
                                     int emit_round, int avg_head);
idfo_stream_i64 *idfo_stream_new_i64(const idfo_layer *layers, int n_layers, int H, int W, int C0,
                                     const int64_t *const *w, const int64_t *const *b,
                                     int emit_round, int avg_head);
void idfo_stream_free_f64(idfo_stream_f64 *);
void idfo_stream_free_i64(idfo_stream_i64 *);

/* Present n_rows rows ([n_rows][W][C0]) one after the other, each pushed through
 * every layer it can influence before the next is looked at.  Returns 0, or -2
 * if a ring slot was needed while it still held an unfinished row (the
 * K_h-rows-per-layer bound would have been violated). */
int idfo_stream_push_f64(idfo_stream_f64 *, const double *rows, int n_rows);
int idfo_stream_push_i64(idfo_stream_i64 *, const int64_t *rows, int n_rows);

/* Rows of the last layer completed and not yet taken. */
int64_t idfo_stream_ready_f64(const idfo_stream_f64 *);
int64_t idfo_stream_ready_i64(const idfo_stream_i64 *);
/* Move up to max_rows completed rows ([n][W_o][C_o]) to out; returns n. */
int64_t idfo_stream_take_f64(idfo_stream_f64 *, double *out, int64_t max_rows);
int64_t idfo_stream_take_i64(idfo_stream_i64 *, int64_t *out, int64_t max_rows);

/* Per-layer counters (arrays of n_layers):
 *   events_in     non-zero values delivered to the layer (pool layers: non-zero inputs)
 *   macs          multiply-adds executed by the layer (conv only)
 *   peak_rows     most rows of the layer held at one moment (ring rows being
 *                 accumulated or in delivery; pool: held row)
 * peak_cells: the most activations held at one moment over the whole net
 * (sum over layers of held rows x W_o x C_out, plus the averaging head's
 * accumulators when present). */
void idfo_stream_stats_f64(const idfo_stream_f64 *, uint64_t *events_in, uint64_t *macs,
                           int *peak_rows, int64_t *peak_cells);
void idfo_stream_stats_i64(const idfo_stream_i64 *, uint64_t *events_in, uint64_t *macs,
                           int *peak_rows, int64_t *peak_cells);

/* Averaging output unit(s) of Fig. 1: running mean over positions of the last
 * layer's emitted activations, one accumulator per channel (avg_head = 1).
 * Returns the number of rows accumulated so far; mean[C_o] filled. */
int64_t idfo_stream_head_f64(const idfo_stream_f64 *, double *mean);
int64_t idfo_stream_head_i64(const idfo_stream_i64 *, double *mean);

#ifdef __cplusplus
}
#endif
#endif
