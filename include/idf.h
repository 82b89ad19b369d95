/*
 * idf -- incremental depth-first CNN inference on one AMD MI355X (gfx950).
 *
 * C ABI of the streaming core described in Binas & Bengio, "Low-memory
 * convolutional neural networks through incremental depth-first processing":
 * input arrives in small segments (single samples of a 1-D signal, rows of an
 * image); every non-zero value of a segment is an event that is added,
 * weighted, into the stateful pre-activations c of every convolution layer it
 * can influence (Sec. 3: stateful neuron, event definition, event-delivery
 * rule); a row of c that no future input can change is activated, emitted to
 * the next layer and forgotten, so each layer keeps only a rolling buffer of
 * K_h rows (Sec. 3 last two paragraphs, Fig. 1, Fig. 2): constant state for
 * 1-D input, state proportional to the row width for 2-D input.  The result
 * equals the conventional layer-by-layer network (Sec. 1, Sec. 4, Sec. 5).
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the GPU that is current when idf_open_streams is called.
 *   - The library never allocates or frees device memory: the caller hands in
 *     one workspace (size from idf_query_sizes) and keeps it alive until
 *     idf_close_streams.
 *   - All device work is enqueued on the hipStream_t given to idf_open_streams
 *     and is asynchronous to the host; calls return after enqueueing.
 *   - Layouts are row-major with channels last: rows [row][x][channel].
 *     1-D signals use in_w = 1, k_w = 1; the streaming axis is always "row".
 *   - Every function returns IDF_OK (0) or a negative IDF_E* code and never
 *     throws or aborts; idf_last_error() gives the text for the calling thread.
 *     On any error nothing has been enqueued.
 *   - A handle must not be used from two threads at once.
 */
#ifndef IDF_H
#define IDF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct idf_net idf_net;          /* immutable network: layers + packed weights (host side) */
typedef struct idf_streams idf_streams;  /* B independent streams of one net on one GPU            */

enum { IDF_OK = 0, IDF_EINVAL = -1, IDF_ENOMEM = -2, IDF_ESTATE = -3, IDF_EDEVICE = -4, IDF_EUNSUPPORTED = -5 };

/* Arithmetic of a network.
 *   IDF_PREC_F32   input, weights, events, state and output are float32.
 *   IDF_PREC_BF16  input, weights and the events passed between layers are bfloat16 (16-bit
 *                  patterns, events rounded to nearest-even when emitted); state c is float32;
 *                  the last layer's output is float32, not rounded.
 *   IDF_PREC_I8    input, weights and events are int8; state c and bias are int32; output int32.
 */
enum { IDF_PREC_F32 = 0, IDF_PREC_BF16 = 1, IDF_PREC_I8 = 2 };

enum { IDF_CONV = 0, IDF_MAXPOOL = 1 };

/* f of the stateful neuron h^ = f(c) (Sec. 3).  All have f(0) = 0, as the paper assumes.
 *   IDF_ACT_RELU_SHR_CLAMP (IDF_PREC_I8 only): min(clamp_hi, max(c, 0) >> shr). */
enum { IDF_ACT_NONE = 0, IDF_ACT_RELU = 1, IDF_ACT_RELU_SHR_CLAMP = 2 };

typedef struct {
    int kind;          /* IDF_CONV | IDF_MAXPOOL (window 2 rows x k_w columns, stride = window, no padding) */
    int c_in, c_out;   /* pool: equal */
    int k_h, k_w;      /* conv: any >= 1.  pool: k_h = 2 and k_w in {1, 2} */
    int s_h, s_w;      /* conv: any >= 1.  pool: s_h = 2, s_w = k_w */
    int p_h, p_w;      /* zero padding, same amount on both sides.  pool: 0 */
    int act;           /* IDF_ACT_* (conv only) */
    int shr, clamp_hi; /* parameters of IDF_ACT_RELU_SHR_CLAMP */
} idf_layer;

typedef struct {
    int precision;     /* IDF_PREC_* */
    int in_h;          /* rows per sample; after row in_h-1 every layer completes its remaining rows
                          (bottom padding) and the stream starts the next sample at row 0.
                          0 = unbounded stream: then every p_h must be 0. */
    int in_w, in_c;    /* row width and channels of the network input */
    int n_layers;
    const idf_layer *layers;   /* host */
} idf_net_desc;

typedef struct {
    size_t workspace_bytes;          /* device memory idf_open_streams needs                        */
    size_t weights_bytes;            /* of which: packed weights and biases (shared by all streams) */
    size_t state_bytes_per_stream;   /* of which, per stream: the retained state -- the rolling rows of
                                        c of every conv layer and the held row of every pool.  This is
                                        the footprint the paper bounds; it does not depend on in_h.  */
    size_t handover_bytes_per_stream;/* of which, per stream: rows a layer has completed that may wait, when a
                                        call returns, for the next layer's step in a later call.  Only the
                                        staged modes have such rows (the default for nets served by the
                                        1-D cascade or throughout by the matrix-core kernel: layer l then
                                        runs behind layer l-1 by one launch); 0 when the layers run strictly
                                        depth-first within every call (environment IDF_CASCADE_STAGES=1,
                                        IDF_NO_ROW_STAGES=1).  Independent of in_h as well.              */
    size_t retained_bytes_per_stream;/* state_bytes_per_stream + handover_bytes_per_stream: everything of a
                                        stream that survives from one call to the next                  */
    size_t transit_bytes_per_stream; /* per stream: room for rows passed between layers (scratch during a
                                        push; also where the hand-over rows above wait)                  */
    size_t output_bytes_per_stream;  /* per stream: completed rows waiting for idf_read_outputs      */
    int    out_w, out_c;             /* shape of one output row                                      */
    int64_t out_h;                   /* output rows per sample (0 if unbounded)                      */
} idf_sizes;

/* Build a network.
 *   weights[i] (host): for conv layer i an array [c_out][c_in][k_h][k_w] of float32 (F32),
 *                      bfloat16 bit patterns as uint16 (BF16) or int8 (I8); ignored for pools.
 *   biases  (host):    NULL, or per layer NULL / [c_out] float32 (F32, BF16) or int32 (I8).  A row
 *                      of c starts at the bias; NULL is the bias-free case the paper restricts
 *                      itself to in Sec. 3.
 * Everything is copied and repacked; the caller keeps ownership of its arrays.
 * IDF_EINVAL: inconsistent description (channel chain, kernel larger than its input, pool shape,
 *             padding on an unbounded stream, unknown enum).  IDF_EUNSUPPORTED: a valid network
 *             this build cannot run (shr/clamp activation outside I8). */
int idf_create_net(const idf_net_desc *desc, const void *const *weights, const void *const *biases,
                   idf_net **out);
/* The same network presented column by column (Fig. 2: the input may arrive row by row or column
 * by column; Sec. 3: any order of small segments): desc, weights and biases describe the network in
 * image coordinates exactly as for idf_create_net, with in_w = 0 allowed for an unbounded number of
 * columns (then every p_w must be 0) and in_h > 0 required.  The returned network streams along the
 * other axis -- everything that says "row" for it means a column of the image:
 *   idf_push_segment takes the next n_rows columns, dev_rows [n_ids][n_rows][in_h][in_c];
 *   idf_read_outputs hands over completed columns of the output map, [n_ids][max_rows][out rows][out_c]
 *   (idf_sizes: out_h = columns per sample, out_w = rows of the output map);
 *   the retained state is proportional to the column length instead of the row width.
 * The values are those of the conventional network, as for row-wise presentation.  Pools must be
 * 2 x 2 (a 2 x 1 pool has no column-wise counterpart here: IDF_EINVAL). */
int idf_create_net_columnwise(const idf_net_desc *desc, const void *const *weights, const void *const *biases,
                              idf_net **out);
/* A network over volumes [slab][row][column][channel] presented slab by slab (Sec. 3 names inputs of
 * more than two dimensions as a further case of the same scheme: the rolling buffer of a layer then
 * holds k_d slabs of c, and a slab is emitted once no later slab can change it).  All layers are
 * convolutions.
 *   weights[i] (host): [c_out][c_in][k_d][k_h][k_w], element type as for idf_create_net;
 *   biases as for idf_create_net.
 * The returned network is used like any other, with "row" meaning slab:
 *   idf_push_segment takes the next n_rows slabs, dev_rows [n_ids][n_rows][in_h][in_w][in_c];
 *   idf_read_outputs hands over completed slabs [n_ids][max_rows][out rows][out columns][c_out]
 *   (idf_sizes: out_h = slabs per sample, out_w = rows of a slab, out_c = columns x channels);
 *   the retained state is k_d slabs per layer, whatever the number of slabs.
 * How it is served: the column axis is folded into the channels (a slab row of in_w x c_in values is
 * one position with in_w * c_in channels; the weights become banded over that axis), so the two
 * streaming axes slab and row run on the kernels of the 2-D case and the values are those of the
 * conventional 3-D network.  The multiply-add counters of idf_get_stats count what those kernels
 * execute per event, i.e. they include the zero entries of the band: (columns of the layer's
 * output) x c_out per tap instead of (taps along the column axis) x c_out.
 * IDF_EINVAL as for idf_create_net; IDF_EUNSUPPORTED if a folded layer is wider than the kernels
 * take (in_w * c_in or out columns * c_out too large). */
typedef struct {
    int c_in, c_out;
    int k_d, k_h, k_w;
    int s_d, s_h, s_w;
    int p_d, p_h, p_w; /* zero padding, same amount on both sides of an axis */
    int act;           /* IDF_ACT_* */
    int shr, clamp_hi; /* parameters of IDF_ACT_RELU_SHR_CLAMP */
} idf_volume_layer;
typedef struct {
    int precision;     /* IDF_PREC_* */
    int in_d;          /* slabs per sample (> 0) */
    int in_h, in_w, in_c;
    int n_layers;
    const idf_volume_layer *layers;   /* host */
} idf_volume_desc;
int idf_create_net_volume(const idf_volume_desc *desc, const void *const *weights, const void *const *biases,
                      idf_net **out);
int idf_destroy_net(idf_net *net);

/* Sizes for n_streams streams that are pushed at most max_seg_rows rows per call and may hold up
 * to out_cap_rows completed output rows per stream between reads (0 = one whole sample; must be
 * > 0 for an unbounded net). */
int idf_query_sizes(const idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows,
                    idf_sizes *out);

/* Open n_streams streams, all at row 0 with zero state (Sec. 3 assumes the network starts
 * from all-zero state).  dev_workspace (device, 256-byte aligned, >= workspace_bytes) stays owned by
 * the caller.  hip_stream: a hipStream_t (NULL = the default stream).  Enqueues the upload of
 * the packed weights. */
int idf_open_streams(idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows,
                     void *dev_workspace, size_t workspace_bytes, void *hip_stream,
                     idf_streams **out);
int idf_close_streams(idf_streams *s);

/* idf_open_streams for callers that cannot allocate device memory at all (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same call without the
 * workspace arguments.  The workspace -- packed weights, rolling buffers, rows between layers,
 * output area, counters -- is an array of IDF_STATIC_WORKSPACE_BYTES bytes inside the library
 * itself, one per GPU, held by every GPU the library runs on until the process ends; neither this
 * call nor anything the returned streams do allocates or frees device memory.  Inputs and outputs
 * are still the caller's (idf_push_segment, idf_read_outputs).
 *   - The array belongs to the GPU that is current at the call.  It keeps what the previous
 *     streams left in it; this call clears every byte it lays out before anything reads it.
 *   - One set of streams per GPU can hold it at a time: IDF_ESTATE while another set opened this
 *     way on the same GPU has not been closed (two sets would race for the same bytes).
 *   - IDF_ENOMEM with the sizes in the message if idf_query_sizes(...).workspace_bytes exceeds
 *     IDF_STATIC_WORKSPACE_BYTES: nothing is opened.
 * Everything else is as for idf_open_streams; close with idf_close_streams. */
#define IDF_STATIC_WORKSPACE_BYTES (32u << 20)
int idf_open_streams_static(idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows,
                            void *hip_stream, idf_streams **out);

/* Present the next n_rows rows to n_ids streams and push them depth-first through every layer
 * they can influence (Sec. 3 first paragraph; Sec. 5, the method seen as a core that takes input
 * as it arrives).
 *   stream_ids (host): n_ids distinct ids in [0, n_streams), or NULL for 0 .. n_ids-1.
 *   dev_rows (device): [n_ids][n_rows][in_w][in_c] in the input type; entry i belongs to
 *                      stream_ids[i].  It is read by the enqueued kernels: keep it unchanged
 *                      until the work has run (stream order).
 *   1 <= n_rows <= max_seg_rows.
 * Zero values are not events: they cause no arithmetic (Sec. 1).  Completed rows of the last
 * layer are appended to the stream's output area.
 * For 1-D nets the deeper layers of a segment may be enqueued only with the next pushes (layers
 * run in stages side by side, each stage on the segment one push older); idf_read_outputs,
 * idf_get_stats, idf_reset_streams, idf_close_streams and idf_profile_end first enqueue whatever
 * is still on its way, so what they return is always the result of every pushed row having gone
 * through every layer it can influence.  The last segment's dev_rows is read by the push itself.
 * For 2-D nets served throughout by the matrix-core kernel a push of all streams in step is one
 * launch per row -- or, when the push brings several rows (streams opened with max_seg_rows >= 2),
 * one launch per two rows: a layer that finds two rows waiting takes both in one step and keeps
 * the rows of c between them on chip instead of writing them to its rolling buffer and reading
 * them back; values and counters are those of a launch per row, bit for bit (environment
 * IDF_NO_ROW_PAIRS=1 switches it off).
 * IDF_EINVAL: bad id, duplicate id, n_rows out of range.  IDF_ESTATE: the rows would run past row
 * in_h-1 of the current sample, or the completed output rows would not fit the output area
 * (read first). */
int idf_push_segment(idf_streams *s, const int32_t *stream_ids, int n_ids, const void *dev_rows,
                     int n_rows);

/* Throughput mode for 1-D nets whose streams are pushed in step (idf_push_segment with all streams
 * at the same row): up to k such segments are held back and run by one launch.  A workgroup takes
 * its stream's held-back segments in order, consecutive ones together while their rows fit one
 * step of a layer (16 rows), with the rolling buffers staying on chip in between; every segment
 * still goes through everything it can influence before the next is looked at (Sec. 3 first
 * paragraph).  k = 1 (the default) launches with every push.
 *   - A held-back segment's dev_rows is read when its launch runs: keep it unchanged until k - 1
 *     further pushes in step or any of the calls below have been made AND the stream's work has run.
 *   - idf_read_outputs, idf_get_stats, idf_get_issued_macs, idf_reset_streams, idf_snapshot,
 *     idf_restore, idf_read_head*, idf_close_streams, idf_profile_end, this call, and any push that is
 *     not of all streams in step first launch what is held back: what they return never shows it.
 *   - Rows of segments taken together are added in one pass: the float32 sums are associated
 *     differently than with a launch per push, so results agree with k = 1 to rounding, not bit for bit.
 *   - A launch is also due as soon as a further segment could make some layer need more than 8 steps.
 * 1 <= k <= 16.  IDF_EUNSUPPORTED for nets the 1-D cascade does not serve and under eager emission. */
int idf_set_push_batching(idf_streams *s, int k);

/* Present the next n_px pixels of the current row (Sec. 3: segments can be arbitrarily small, down
 * to single components): columns x0 .. x0+n_px-1, in order -- x0 must be the stream's next column.
 *   dev_pixels (device): [n_ids][n_px][in_c] in the input type.
 * The pixels are taken into the first layer's rolling buffer at once; rows can only become final,
 * and the deeper layers fire, with the segment that makes the row whole (x0 + n_px == in_w), which
 * then does everything a pushed row does.  A row begun this way must be finished this way.
 * Any convolution can be the first layer (any kernel size, stride and padding, all precisions).
 * IDF_EUNSUPPORTED when the first layer is a pool, and under eager emission; IDF_ESTATE: x0 is not
 * the next column. */
int idf_push_pixels(idf_streams *s, const int32_t *stream_ids, int n_ids, const void *dev_pixels, int x0,
                    int n_px);

/* Hand over the output rows completed since the previous read.
 *   dev_out (device): [n_ids][max_rows][out_w][out_c] float32 (F32, BF16) or int32 (I8); for
 *                     stream i rows 0 .. n_rows[i]-1 are written.
 *   first_row, n_rows (host, length n_ids): index of the first row within its sample, and how
 *                     many rows.  These follow from the number of rows pushed alone (the schedule
 *                     does not depend on the data), so no device synchronisation happens here; the
 *                     copy itself is enqueued on the stream.
 * At most max_rows rows per stream are taken; the rest stay for the next read. */
int idf_read_outputs(idf_streams *s, const int32_t *stream_ids, int n_ids, void *dev_out,
                     int64_t max_rows, int64_t *first_row, int32_t *n_rows);

/* Forget everything about these streams (state, pending output): next row is row 0. */
int idf_reset_streams(idf_streams *s, const int32_t *stream_ids, int n_ids);

/* Counters of one stream since open/reset, per layer (host arrays of n_layers; any may be NULL):
 *   events_in      non-zero values delivered to the layer
 *   macs_executed  multiply-adds those events caused (taps landing inside the layer's output
 *                  x c_out); 0 for pools
 *   state_bytes    retained state of the layer for one stream
 * Synchronises the stream. */
int idf_get_stats(idf_streams *s, int stream_id, uint64_t *events_in, uint64_t *macs_executed,
                  uint64_t *state_bytes);

/* Multiply-adds the kernels issued for one stream, per layer (host array of n_layers): what the
 * compaction of events (Sec. 1: zero values cause no arithmetic) leaves over.  Counted only while
 * switched on with idf_count_issued_macs(s, 1) (off after open: the count costs an atomic per
 * wave), since open/reset.
 * The matrix-core kernel skips K-steps whose 32-position fragment holds no event and multiplies
 * the zeros inside the others (a first layer of 1-4 input channels has one or two K-steps and
 * visits them always); the 1-D cascade skips input channels without an event in the
 * segment and computes all rows of the others; layers served by the generic kernels, which test
 * every value, report their executed count.  Counted from open/reset on it is always >=
 * macs_executed of idf_get_stats.  IDF_EUNSUPPORTED under eager emission.  idf_get_issued_macs
 * synchronises the stream. */
int idf_count_issued_macs(idf_streams *s, int on);
int idf_get_issued_macs(idf_streams *s, int stream_id, uint64_t *macs_issued);

/* Event-list variant of the int8 matrix-core kernel (Sec. 1 and Sec. 3: work in proportion to the
 * events, one visit per event and tap).  A tile whose stretch holds at most events_per_kstep events
 * per K-step of its contraction (and at most 256 in all; a first layer of 1-4 input channels: at
 * most 256) packs them into a list in LDS and visits them on the vector units -- three multiply-adds
 * per event and output channel -- instead of contracting; layers of more than 16 input channels and
 * the other precisions always contract.  The sums are the same integers either way, so outputs do
 * not change bit for bit; only idf_get_issued_macs and the time do.  0 (the setting after open)
 * switches it off: on MI355X one K-step of the contraction costs a wave less than the visit of a
 * single event's three taps for 32 channels, so the list only pays below about one event per 16
 * positions and channels, far sparser than rectified feature maps are.  Takes effect for segments
 * pushed after the call (drains what is on its way).  IDF_EUNSUPPORTED under eager emission. */
int idf_set_event_path(idf_streams *s, int events_per_kstep);

/* Rows of the current sample a stream has been given so far (host bookkeeping, no device work). */
int idf_rows_pushed(const idf_streams *s, int stream_id, int64_t *rows);

/* Eager emission -- Sec. 3 taken literally: every neuron announces a change of f(c) at once, as an
 * event that the next layer takes in at once, so that after every pushed segment the announced
 * activations of every layer are those of the conventional network on the input seen so far (the
 * rest taken as zero; Sec. 4, Fig. 3).  State lives in a second caller-owned device workspace of
 * idf_query_eager_bytes() bytes; bounded samples only (IDF_EUNSUPPORTED otherwise); all three
 * precisions (a bfloat16 net announces values rounded to bfloat16, the last layer unrounded, like
 * its row-complete counterpart).
 *   Nets without biases keep, per stream and level, only the rows that a future segment can still
 *   change or that a pool still looks at -- the cone of Sec. 3: 1 + n(K-1) rows plus the segment at
 *   depth n for K x K layers of stride 1 -- in a ring, so that the state does not depend on the sample
 *   height; only the last level's announced map, the output, is kept whole.  A net with biases keeps
 *   every level whole: every neuron announces f(bias ...) before any input arrives (Sec. 3 assumes
 *   b = 0 for exactly this reason).
 * After idf_enable_eager (before the first push) idf_push_segment delivers eagerly, idf_read_outputs
 * is refused (IDF_ESTATE) and
 *   idf_read_announced(level, ...) copies the announced map [n_ids][H][W][C] of 4-byte values of a
 *     level that is kept whole -- the last level (n_layers) always, any level (0 = the input) of a net
 *     with biases -- to dev_out, in stream order (IDF_ESTATE for a level kept as a ring);
 *   idf_read_announced_rows(level, ...) copies the rows of a level that are still kept, oldest first,
 *     to dev_out [n_ids][max_rows][W][C] and reports per stream the index of the first and how many
 *     (at most max_rows).  Rows before them are final and forgotten, rows after them still all zero.
 * idf_get_stats then counts, per layer, the non-zero changes delivered to it.
 * idf_eager_state_bytes: state c and announced values retained per stream (without the output map);
 * rows_kept (host, n_layers + 1 entries, may be NULL): rows kept per level. */
int idf_query_eager_bytes(const idf_net *net, int n_streams, int max_seg_rows, size_t *bytes);
int idf_enable_eager(idf_streams *s, void *dev_workspace, size_t workspace_bytes);
int idf_read_announced(idf_streams *s, int level, const int32_t *stream_ids, int n_ids, void *dev_out);
int idf_read_announced_rows(idf_streams *s, int level, const int32_t *stream_ids, int n_ids, void *dev_out,
                            int max_rows, int64_t *first_row, int32_t *n_rows);
int idf_eager_state_bytes(const idf_streams *s, size_t *per_stream, int *rows_kept);

/* Averaging output units (Fig. 1: the output neuron that averages the last layer; Sec. 4: output
 * units whose value converges as rows come in): one accumulator per channel of the last layer,
 * fed by the rows the last layer completes; the value is the running mean over the positions of
 * the rows completed so far in the current sample (a bounded net starts anew with the first row
 * of the next sample).  Accumulation is in float64 (exact for int32 outputs).
 * idf_enable_head: before the first push after open (IDF_ESTATE otherwise).
 * idf_read_head: mean (host) [n_ids][out_c], rows (host) [n_ids] = rows averaged.  Synchronises
 * the stream.  IDF_ESTATE if the head was not enabled. */
int idf_enable_head(idf_streams *s);
int idf_read_head(idf_streams *s, const int32_t *stream_ids, int n_ids, double *mean, int64_t *rows);

/* The retained state of one stream -- what the recurrent view of Sec. 5 would call the hidden state: rolling
 * buffers of c of every conv layer, held rows of the pools, the counters of idf_get_stats, the
 * averaging units, and where the stream stands -- copied to / from a caller-owned device buffer
 * of idf_snapshot_bytes() bytes.  A snapshot can be restored into any stream of the same set of
 * open streams: that stream continues exactly where the snapshot was taken; what it held before
 * is gone.  Both need the stream's completed output rows to have been read (IDF_ESTATE otherwise);
 * both are enqueued on the stream like a push. */
typedef struct {
    int64_t rows_pushed;      /* rows of the current sample received */
    int64_t out_rows;         /* output rows completed (and read) since open / reset */
    int64_t head_rows;        /* rows the averaging units hold */
} idf_stream_pos;
int idf_snapshot_bytes(const idf_streams *s, size_t *bytes);
int idf_snapshot(idf_streams *s, int stream_id, void *dev_buf, idf_stream_pos *pos);
int idf_restore(idf_streams *s, int stream_id, const void *dev_buf, const idf_stream_pos *pos);

/* Fully connected output units over the last layer's map (Sec. 4: the class units whose values
 * settle as rows come in, Fig. 3 / Fig. 4): unit k holds bias[k] plus the sum, over the rows the
 * last layer has completed in the current sample, of weights[k][row][x][c] times the activation
 * -- every non-zero activation is an event delivered to every unit (Sec. 3).  float64 sums.
 *   weights (host) [n_units][out_h][out_w][out_c] float32, bias (host) [n_units] or NULL: copied.
 *   dev_buf (device): idf_query_head_units_bytes() bytes, owned by the caller, kept by the streams.
 * Enabling also enables the averaging units and has the same precondition (before the first push);
 * bounded samples only (IDF_EUNSUPPORTED otherwise).
 * idf_read_head_units: values (host) [n_ids][n_units], rows (host) [n_ids]; synchronises. */
int idf_query_head_units_bytes(const idf_net *net, int n_streams, int n_units, size_t *bytes);
int idf_enable_head_units(idf_streams *s, int n_units, const float *weights, const float *bias, void *dev_buf,
                          size_t bytes);
int idf_read_head_units(idf_streams *s, const int32_t *stream_ids, int n_ids, double *values, int64_t *rows);

/* Which kernel family serves layer i of an open stream set: a short static name such as
 * "generic", for reports.  NULL on a bad index. */
const char *idf_layer_kernel(const idf_streams *s, int layer);

/* Kernel timing, for benchmarks and reports (the paper gives no timings; this is how the build
 * measures itself).  Between idf_profile_begin and idf_profile_end every kernel the library
 * launches for this stream set is bracketed by a HIP event pair that the runtime stamps at the
 * kernel's own start and end.  idf_profile_end synchronises the stream and returns, per kernel
 * family and layer (name "family@layer"; families that span the whole net have no "@layer"), the
 * number of launches, the summed execution time and the summed algorithmic bytes (network input
 * read, retained state read and written, weights once per launch, output rows written).
 * out: host array of max_kinds entries; *n_kinds receives how many were filled. */
typedef struct {
    char name[32];
    uint64_t launches;
    double total_ms;
    double algorithmic_bytes;
} idf_kernel_profile;
int idf_profile_begin(idf_streams *s);
int idf_profile_end(idf_streams *s, int max_kinds, idf_kernel_profile *out, int *n_kinds);

/* What this machine delivers to a plain kernel, to be quoted next to the published peaks that
 * the rooflines are priced against (for benchmarks and reports; nothing on the streaming path
 * calls it, and the paper names no hardware).  kind selects the kernel:
 *   IDF_PEAK_COPY       copies the first half of dev_buf to the second half in 16-byte pieces;
 *                       *rate = bytes read + written per second, in GB/s.  Use a buffer well
 *                       beyond the last-level cache (1 GiB or more) to see the memory itself.
 *   IDF_PEAK_FMA_F32    independent chains of float32 multiply-adds on the vector units;
 *   IDF_PEAK_MFMA_F32 / _BF16 / _I8   independent chains of the 32x32x2 float32, 32x32x16
 *                       bfloat16 and 32x32x32 int8 matrix instructions, on every compute unit;
 *                       *rate = operations per second (multiply and add counted separately), in
 *                       tera-operations/s.
 * dev_buf: device memory of at least 1 MiB (written); hip_stream: the hipStream_t to run on.
 * The call launches the kernel once untimed and three times timed by HIP events stamped at the
 * kernel's own start and end, synchronises the stream and reports the fastest of the three.
 * Errors: IDF_EINVAL (null pointer, unknown kind, buffer too small), IDF_EDEVICE. */
enum { IDF_PEAK_COPY = 0, IDF_PEAK_FMA_F32 = 1, IDF_PEAK_MFMA_F32 = 2, IDF_PEAK_MFMA_BF16 = 3, IDF_PEAK_MFMA_I8 = 4 };
int idf_measure_peak(int kind, void *dev_buf, size_t bytes, void *hip_stream, double *rate);

const char *idf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
