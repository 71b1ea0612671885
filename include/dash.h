/*
 * dash.h -- C ABI of libdash: garbling and evaluating arithmetic garbled circuits over CRT
 * residues on one AMD MI355X (gfx950), after "Dash" (arXiv 2302.06361).
 *
 * The four scheme algorithms of the paper (Sec. Garbled Circuits: Gb, En, Ev, De) map to
 *   Gb : dash_input_labels + dash_garble_layer per layer      En : dash_encode
 *   Ev : dash_eval_layer per layer                            De : dash_decode
 *
 * Conventions that hold for every entry point
 *   - "device" pointers are HIP device memory on the context's GPU, owned by the caller;
 *     "host" pointers are ordinary host memory.  The library owns only the dash_ctx.
 *   - Calls enqueue work on the given hipStream_t (passed as void*, NULL = default stream) and
 *     return without synchronising; no call allocates or frees device memory except
 *     dash_ctx_create / dash_ctx_destroy.
 *   - Return value: 0 = DASH_OK, negative = error (dash_strerror).  Nothing is launched when an
 *     argument check fails.  A forged output label is data (valid[] of dash_decode), not an error.
 *
 * LabelTensor layout (the paper's LabelTensor, Sec. LabelTensors, re-laid out for 64-wide
 * wavefronts): one tensor per CRT residue; the lambda digits of a label (one byte each, values
 * in [0, p)) are cut into chunks of 16 digits and the tensor is stored chunk-major,
 *      digit j of element e  at  data + (j / 16) * chunk_stride + 16 * e + (j % 16),
 * so consecutive elements of one chunk are consecutive 16-byte words (one dwordx4 per lane,
 * fully coalesced) and, inside a batch element, consecutive features are consecutive words (the
 * K-contiguous operand of the int8 MFMA contraction).  Digits past lambda in the last chunk are
 * zero.  Elements are ordered [batch][y][x][channel].
 *
 * Ciphertext tables (Sec. Arithmetic Garbled Circuits, projection gates: p ciphertexts per gate,
 * ordered by the colour = digit 0 of the input label): a batch of E gates Z_p -> Z_q is one
 * segment [gate][row 0..p-1][pitch_q] with pitch_q = 4 * ceil(lambda_q / 4) bytes, pad bytes
 * zero.  A layer's table buffer is the concatenation of its segments in slot order; segment s
 * starts at E * (bytes per element of the segments before s).
 */
#ifndef DASH_H
#define DASH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DASH_MAX_PRIMES 16
#define DASH_MAX_DIGITS 16

enum {
    DASH_OK = 0,
    DASH_EINVAL = -1,       /* bad argument (NULL, out of range, inconsistent shapes) */
    DASH_ESIZE = -2,        /* a size exceeds what the kernels support */
    DASH_EHIP = -3,         /* a HIP runtime call failed */
    DASH_EUNSUPPORTED = -4  /* valid request that this build does not implement */
};

/* Label length rule (Sec. LabelTensors, figure caption).  CEIL: smallest lambda with
 * m^lambda >= 2^128 (at least 128 bits per label).  FLOOR: largest lambda with m^lambda <= 2^128
 * (the caption's floor(128 / log2 m): the label packs into one 128-bit block). */
enum { DASH_LAMBDA_CEIL = 0, DASH_LAMBDA_FLOOR = 1 };

enum {
    DASH_DENSE = 1,    /* out[j] = sum_i W[j][i] * in[i] (+ bias[j])           free gates  */
    DASH_CONV2D = 2,   /* 2-d convolution, zero padding, square stride          free gates  */
    DASH_SUMPOOL = 3,  /* 2x2 sum, stride 2                                     free gates  */
    DASH_RELU = 4,     /* a * sgn_{0,1}(a): sign gadget + mixed-modulus half gates           */
    DASH_SCALE = 5,    /* CRT scaling by 2, `repeat` times                                  */
    DASH_SIGN = 6,     /* sgn_{-1,1}(a)                                                     */
    DASH_PROJ = 7      /* n independent unary gates Z_p -> Z_q with per-gate function tables */
};

typedef struct dash_ctx dash_ctx;

/* One LabelTensor per CRT residue (see the layout above). */
typedef struct {
    void *data[DASH_MAX_PRIMES];            /* device */
    int64_t chunk_stride[DASH_MAX_PRIMES];  /* bytes between chunks, >= 16 * n_elem, multiple of 16 */
    int64_t n_elem;
} dash_labels;

/* One layer call.  Fields not used by `kind` are ignored. */
typedef struct {
    int32_t kind;
    int32_t layer_id;   /* 0..65535, enters every hash tweak and PRG counter of the layer */
    int64_t elem_base;  /* index, inside the whole layer, of this call's element 0: a layer may be
                           processed in several calls over disjoint element ranges (batch chunks) */
    int64_t n_elem;     /* RELU / SCALE / SIGN / PROJ: values (gates) in this call;
                           DENSE / CONV2D / SUMPOOL: batch elements in this call */
    /* DENSE (in_c = K inputs, out_c = M outputs), CONV2D, SUMPOOL (in_h, in_w, in_c) */
    int32_t in_h, in_w, in_c, out_c, kh, kw, stride, pad;
    const void *weights;  /* device, written by dash_weights_prepare */
    const int32_t *bias;  /* device int32 [out_c] or NULL: added as bias * (constant-one wire) */
    /* SCALE */
    int32_t repeat;
    /* PROJ: input tensor in->data[p_index], output tensor out->data[q_index] */
    int32_t p_index, q_index;
    const uint8_t *phi;   /* device, function tables, phi[g * phi_stride + a] in [0, q) */
    int64_t phi_stride;   /* p (one table per gate) or 0 (one table for all gates) */
} dash_layer;

/* Create a context on GPU `hip_device`: the CRT base (distinct primes, primes[0] must be 2 for
 * SCALE, every prime <= 127, product of the primes below 2^62), the label lengths, the 16-byte seed of
 * the counter-based PRG that replaces the paper's hardware RNG (Sec. Implementation) and the
 * mixed-radix digits d_1..d_n of the sign gadget (Appendix, Approximated Garbled Sign; d_1 most
 * significant and even, k * d_j <= 255; NULL = built-in set with prod(d) >= k * P, which makes the
 * sign exact).
 * Label lengths (Sec. LabelTensors): lambda_rule gives the length of every modulus; `lambda`, if not
 * NULL, is a host array of k entries that overrides it for the CRT primes (lambda[i] digits for
 * primes[i], 1..128; the accumulation moduli of the sign gadget keep the rule).
 * Draws the offset label R_m of every modulus in use (colour digit forced to 1) and the
 * constant-one wire of every prime.  Allocates a few hundred KB of device memory.  Tuning variables of
 * the environment (DASH_BANKED_MIN_LANES, DASH_DIGITS_BANKED_MIN_LANES, DASH_FUSED_MIN_ELEMS_GARBLE,
 * DASH_FUSED_MIN_ELEMS_EVAL, DASH_GEMM_TILE) are read here, once per context, and nowhere else.
 * Errors: DASH_EINVAL (NULL, non-prime or repeated modulus, bad digits or lambda), DASH_ESIZE (product
 * of the primes too large), DASH_EUNSUPPORTED (no digit set found), DASH_EHIP. */
int dash_ctx_create(dash_ctx **out, const uint16_t *primes, int k, int lambda_rule, const uint16_t *lambda,
                    const uint8_t seed[16], const uint16_t *sign_digits, int n_digits, int hip_device);
void dash_ctx_destroy(dash_ctx *ctx);

/* Label length of modulus m (2..255) under the context's rule; 0 if m is out of range. */
int dash_lambda(const dash_ctx *ctx, int m);
/* Copy to host memory: the offset label R_m (lambda_m bytes) of a modulus the context uses;
 * the constant-one wire of prime i (which = 0 zero label, 1 active label).  Synchronous. */
int dash_ctx_offset(const dash_ctx *ctx, int m, uint8_t *host_out);
int dash_ctx_one(const dash_ctx *ctx, int i, int which, uint8_t *host_out);
/* Mixed-radix digits in use: writes d_1..d_n to host_digits (DASH_MAX_DIGITS entries), returns n. */
int dash_ctx_digits(const dash_ctx *ctx, uint16_t *host_digits);

/* Sizes of one layer call: output elements (values, or batch elements for the linear kinds:
 * then *out_elems is values per batch element), bytes of ciphertext tables, bytes of scratch. */
int dash_layer_sizes(const dash_ctx *ctx, const dash_layer *layer, int64_t *out_elems, size_t *table_bytes,
                     size_t *scratch_bytes);

/* Weights of a linear layer are public constants (Sec. Arithmetic Garbled Circuits,
 * multiplication by a public constant): reduce them once per prime into the int8 operand layout
 * of the contraction kernels.  w: device int32 [out_c][K] (K = kh*kw*in_c, order [ky][kx][ci]). */
size_t dash_weights_bytes(const dash_ctx *ctx, int out_c, int K);
int dash_weights_prepare(dash_ctx *ctx, const int32_t *w, int out_c, int K, void *prepared, void *hip_stream);

/* Gb, one layer: from the zero labels of the layer's input wires produce the zero labels of its
 * output wires and (RELU, SCALE, SIGN, PROJ) its ciphertext tables.  Fresh zero labels come from
 * the PRG, addressed by (layer_id, slot, element).  tables / scratch: device, sizes from
 * dash_layer_sizes (may be NULL when the size is 0).  For RELU, SCALE and SIGN out_zero may be the same bundle as in_zero
 * (in place; likewise out_act and in_act of dash_eval_layer); bundles that overlap only in part are not supported. */
int dash_garble_layer(dash_ctx *ctx, const dash_layer *layer, const dash_labels *in_zero, dash_labels *out_zero,
                      void *tables, void *scratch, void *hip_stream);
/* Ev, one layer: from the active labels of the input wires and the tables produce the active
 * labels of the output wires. */
int dash_eval_layer(dash_ctx *ctx, const dash_layer *layer, const dash_labels *in_act, const void *tables,
                    dash_labels *out_act, void *scratch, void *hip_stream);

/* n independent layer calls in one (Sec. LabelTensors: gates of the same kind are processed together as tensors): the
 * result is that of dash_garble_layer (dash_eval_layer) on (layers[i], in[i], out[i], tables[i], scratch[i]) for
 * i = 0 .. n-1, and no call of the list may read what another one writes.  The library may serve several calls with
 * one kernel launch: PROJ calls with the same layer_id and the same output modulus share launches of up to 16 calls
 * (the 144 (p, q) groups of a mixed batch of independent gates take 12 gate launches instead of 144); other kinds are
 * run in turn.  layers, in, out: host arrays of n entries; tables, scratch: host arrays of n device pointers (an entry
 * may be NULL where dash_layer_sizes gives 0; scratch itself may be NULL if no call needs scratch).  If the list holds
 * PROJ calls only, nothing is launched when the argument check of any call fails; otherwise the calls before the
 * failing one have been enqueued. */
int dash_garble_layers(dash_ctx *ctx, int n, const dash_layer *layers, const dash_labels *in_zero, dash_labels *out_zero,
                       void *const *tables, void *const *scratch, void *hip_stream);
int dash_eval_layers(dash_ctx *ctx, int n, const dash_layer *layers, const dash_labels *in_act, const void *const *tables,
                     dash_labels *out_act, void *const *scratch, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops with a fixed memory
 * budget, harnesses that forbid hipMalloc): dash_eval_layer with the scratch buffer taken from a fixed array of
 * DASH_NOALLOC_SCRATCH_BYTES that lives inside the library (one copy per GPU, held until the process ends; its
 * device address is resolved once per GPU by dash_ctx_create).  Same arguments, results and errors as
 * dash_eval_layer otherwise; inputs, tables and outputs are still the caller's.  Returns DASH_ESIZE, and launches
 * nothing, when the layer call needs more scratch than the array holds (dash_layer_sizes reports the need; split
 * the layer into several calls over element ranges then).  The call allocates and frees nothing and does not
 * synchronise.  Every kernel writes the scratch wires it reads, so nothing has to be cleared between calls, but all
 * calls on one GPU share the one array: two calls that may overlap in time on the same GPU (different streams,
 * different contexts) race; order them. */
#define DASH_NOALLOC_SCRATCH_BYTES (32u << 20)
int dash_eval_layer_noalloc(dash_ctx *ctx, const dash_layer *layer, const dash_labels *in_act, const void *tables,
                            dash_labels *out_act, void *hip_stream);

/* e: zero labels of the circuit-input wires first_wire .. first_wire + n - 1, every residue, into elements 0 .. n - 1
 * of `zero` (n <= zero->n_elem, else DASH_EINVAL). */
int dash_input_labels(dash_ctx *ctx, int64_t first_wire, int64_t n, dash_labels *zero, void *hip_stream);
/* En: out = zero + (value mod p) * R_p (Sec. Quantization and Encoding: Encode(x) = x mod P).
 * values: device int64 [n].  A residue whose data pointer is NULL in both bundles is skipped (bundles that carry
 * a single residue, as the inputs of PROJ gates do); NULL in only one of them is DASH_EINVAL. */
int dash_encode(dash_ctx *ctx, const int64_t *values, int64_t n, const dash_labels *zero, dash_labels *out,
                void *hip_stream);
/* De: per element, the residue a_i with act = zero + a_i * R_p on every digit, CRT-reconstructed and
 * mapped to signed (upper half of Z_P negative).  values: device int64 [n]; valid: device u8 [n],
 * 0 where some residue's label is not a valid label of its wire (then values = 0). */
int dash_decode(dash_ctx *ctx, const dash_labels *act, const dash_labels *zero, int64_t n, int64_t *values,
                uint8_t *valid, void *hip_stream);

/* The 128-bit wire format of labels (Sec. Evaluation, online communication: every label is compressed
 * to 128 bits for transfer; Sec. Implementation: compress(l) = (...(l_n p + l_{n-1}) p + ...) p + l_1).
 * packed: device, 16-byte aligned, [k residues][n][16 bytes], each entry the little-endian 128-bit
 * integer sum_j l_j p^j of the label of element e (elements 0 .. n-1 of the LabelTensor), residue i.
 * 16 bytes per label instead of 16 * ceil(lambda / 16).  unpack is the inverse (base-p digits, least
 * significant first, digits past lambda zero).  Lossless only if p^lambda <= 2^128 for every residue,
 * i.e. for contexts created with the floor rule of the LabelTensor figure; otherwise both calls
 * return DASH_EUNSUPPORTED and touch nothing.  Asynchronous on the stream, no allocation. */
int dash_labels_pack(dash_ctx *ctx, const dash_labels *labels, int64_t n, void *packed, void *hip_stream);
int dash_labels_unpack(dash_ctx *ctx, const void *packed, int64_t n, dash_labels *labels, void *hip_stream);

/* The packed storage format of a layer's ciphertext tables, for keeping garbled layers and for shipping them from the
 * garbling device to the inference device (Sec. System-level Architecture, offline phase).  A ciphertext is an
 * encrypted label, a vector in Z_q^lambda, and is compressed exactly like a label (Sec. Implementation, compress;
 * Sec. Evaluation: labels travel as 128 bits): row r of a segment becomes the little-endian 128-bit integer
 * sum_j row[j] q^j, 16 bytes instead of pitch_q = 4 ceil(lambda_q / 4); the one-digit rows of a half gate become one
 * byte each.  Packed layout: the layer's segments in the same order, segment [gate][row][16] (one-digit segments
 * [gate][row][1], padded to a multiple of 16 bytes).  `layer` is the descriptor the tables were garbled with (kind,
 * n_elem, repeat, p_index / q_index).  Lossless only if q^lambda_q <= 2^128 for every output modulus of the layer,
 * i.e. for contexts with the floor rule; otherwise dash_tables_packed_bytes returns 0 and the two calls return
 * DASH_EUNSUPPORTED and touch nothing.  The garbling and evaluating kernels work on the unpacked format: unpack before
 * dash_eval_layer.  tables: device, 4-byte aligned; packed: device, 16-byte aligned, dash_tables_packed_bytes bytes.
 * Asynchronous on the stream, no allocation.  (Garbled row reduction, which would drop one row per gate, is not part
 * of the scheme: Sec. Arithmetic Garbled Circuits, projection gates, leaves it out.) */
size_t dash_tables_packed_bytes(const dash_ctx *ctx, const dash_layer *layer);
int dash_tables_pack(dash_ctx *ctx, const dash_layer *layer, const void *tables, void *packed, void *hip_stream);
int dash_tables_unpack(dash_ctx *ctx, const dash_layer *layer, const void *packed, void *tables, void *hip_stream);

const char *dash_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* DASH_H */
