/*
 * mc.h -- C ABI of libmc: one rank's share of a multi-colour Allreduce step fused with
 * the SGD update, on one AMD MI355X (gfx950).
 *
 * Background (paper: "Efficient Training of Convolutional Neural Nets on Large Distributed
 * Systems", arXiv 1711.00705).  In data-parallel SGD every worker needs the elementwise sum
 * of all workers' gradients (Section 3, Algorithm 1).  The k-colour Allreduce (Section 4.2)
 * cuts the flat gradient payload into k chunks ("colours"), sums each chunk along its own
 * spanning tree, independently of the others, and a rank that is root or inner node of a
 * colour's tree adds what arrived from its children to the contributions of its own GPUs.
 * Each GPU then performs the SGD step with the summed gradient.  This library is that
 * per-rank arithmetic: P staged contributions, packed from per-layer tensors into the flat
 * colour-chunked payload, summed per colour in a fixed sequence, fused with the update.
 *
 * Conventions
 *   - Every function returns an int: MC_OK (0) or a negative MC_ERR_* code.  No C++ type,
 *     exception or torch type crosses this boundary.
 *   - "device" pointers are HIP device addresses valid on the current device; "host"
 *     pointers are ordinary process memory.  All element data is IEEE binary32 ("fp32"),
 *     moved as 32-bit words by pack/unpack and added/multiplied with round-to-nearest-even,
 *     denormals preserved, no fused multiply-add, in reduce_update.
 *   - The caller owns every device buffer and the stream.  The library owns only mc_layout
 *     objects (host tables, plus a small device copy of the offset tables made by
 *     mc_layout_prepare), from create to destroy.  Host arrays passed in are read during
 *     the call and never retained.
 *   - mc_pack / mc_unpack / mc_reduce_update validate their arguments on the host BEFORE
 *     any launch; on error no output is touched.  On success they enqueue work on `stream`
 *     (NULL = the default stream) and return without synchronising.  The exceptions, which
 *     allocate device memory and copy synchronously: mc_layout_prepare, mc_tensor_set_create, and
 *     the first mc_pack / mc_unpack / mc_pack_set / mc_unpack_set / mc_fused_step(_ex) on a device
 *     for a layout that was not prepared there.  Prepare layouts and create tensor sets at set-up
 *     and no later call allocates, copies or blocks.
 *   - After mc_layout_prepare a layout's tables never change and it may be used from several host
 *     threads and streams at once.  (One call counter inside it does change: it only picks the
 *     direction in which MC_SWEEP_AUTO calls walk the payload, see mc_update_spec.)
 *   - What validation cannot see: a device pointer carries no length.  Every flat buffer of a
 *     call must hold the layout's N elements and tensor t of a tensor list numel[t] elements,
 *     all resident on the current device.  Null pointers, misalignment and overlap are
 *     rejected; a buffer that is shorter than stated is not detectable on the host, and the
 *     kernels then read or write past its end (a device memory fault).  The same holds for a
 *     pointer that is not a device address.
 */
#ifndef MC_H_
#define MC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mc_layout mc_layout;        /* opaque */

enum {
    MC_OK = 0,
    MC_ERR_INVALID_ARG = -1,   /* NULL where a pointer is required, count out of range, bad order row */
    MC_ERR_ALIGN = -2,         /* a flat buffer is not 16-byte aligned / a tensor not 4-byte aligned */
    MC_ERR_OVERLAP = -3,       /* two buffers of one call overlap */
    MC_ERR_ALLOC = -4,         /* host allocation failed */
    MC_ERR_HIP = -5,           /* a HIP runtime call failed; see mc_last_hip_error() */
    MC_ERR_LIMIT = -6          /* the input exceeds a fixed capacity of the entry point called */
};

#define MC_MAX_P 32                 /* most contributions one call can sum */
#define MC_COLOUR_ALIGN_ELEMS 256   /* colour chunk length is a multiple of this (1 KiB) */

/* ---- a1: layout --------------------------------------------------------------------
 * Section 4.2 (the payload is split into k chunks, one per colour): the payload is the dense
 * concatenation of the n per-layer tensors in the given order (tensor t occupies flat
 * elements [off_t, off_t + numel[t]), off_t = numel[0] + ... + numel[t-1], N = off_n), and
 * colour c owns flat elements [b_c, b_{c+1}) with b_c = min(N, c*C),
 * C = ceil(N / k) rounded up to MC_COLOUR_ALIGN_ELEMS.  Trailing colours may be empty.
 *
 * numel: host, n_tensors entries, each >= 0 (0 = the tensor occupies nothing).
 * out:   receives the new layout (NULL on failure).  Host-only: touches no GPU.
 * Errors: MC_ERR_INVALID_ARG (NULL, n_tensors < 1, k_colours < 1, negative numel, or a
 * total above 2^40 elements), MC_ERR_ALLOC. */
int mc_layout_create(const int64_t* numel, int32_t n_tensors, int32_t k_colours, mc_layout** out);

/* Frees host tables and any device tables.  NULL is a no-op returning MC_OK. */
int mc_layout_destroy(mc_layout* L);

/* Uploads the offset tables that pack/unpack kernels read to the CURRENT device (one small
 * allocation, one synchronous copy; idempotent).  mc_pack / mc_unpack call it themselves on
 * first use; call it explicitly before capturing a graph or timing.  MC_ERR_HIP on failure. */
int mc_layout_prepare(mc_layout* L);

/* Queries (host outputs).  N: one int64.  off: n_tensors+1 entries.  b: k_colours+1. */
int mc_layout_total(const mc_layout* L, int64_t* N);
int mc_layout_counts(const mc_layout* L, int32_t* n_tensors, int32_t* k_colours);
int mc_layout_tensor_offsets(const mc_layout* L, int64_t* off);
int mc_layout_colour_bounds(const mc_layout* L, int64_t* b);
/* The work items of mc_fused_step: inside colour c, tensor t is cut into runs of 256 elements counted
 * from the tensor's own first element (so that a run's accesses to the per-layer tensors start on a
 * 1 KiB boundary of the tensor, whatever its flat offset); a run cut by a colour bound or by the
 * tensor's end is shorter.  Every colour owns *units_per_colour slots.  unit_tensor (k_colours x
 * units_per_colour entries, or NULL): the tensor of each slot, -1 for an unused one.  unit_first
 * (n_tensors + k_colours entries, or NULL): at c + t, the index within colour c of the first run of
 * tensor t.  *units_per_colour is 0 for layouts without this table (more than 32 colours, an empty
 * payload), which mc_fused_step serves with flat 256-element tiles instead. */
int mc_layout_units(const mc_layout* L, int32_t* units_per_colour, int32_t* unit_tensor, int32_t* unit_first);

/* ---- a2 / a5: pack and unpack ------------------------------------------------------
 * The payload handed to the Allreduce is ONE flat buffer (Section 4.2; Section 5.1 quotes
 * its size), while the framework holds one gradient tensor per layer:
 *   pack:    flat[off_t + j]   = tensors[t][j]      for every t, j < numel[t]
 *   unpack:  tensors[t][j]     = flat[off_t + j]
 * Pure 32-bit word copies: every bit pattern (NaN payloads included) survives.
 *
 * tensors: host array of n_tensors device pointers, each 4-byte aligned, each with
 *          numel[t] readable (pack) / writable (unpack) fp32; entries of zero-length
 *          tensors are ignored and may be NULL.
 * flat:    device, N fp32, 16-byte aligned.
 * Errors: MC_ERR_INVALID_ARG (NULL L / tensors / flat with N > 0 / a NULL entry of a
 * non-empty tensor), MC_ERR_ALIGN, MC_ERR_OVERLAP (a tensor overlaps flat; for unpack also two
 * destination tensors that overlap each other), MC_ERR_HIP. */
int mc_pack(mc_layout* L, const void* const* tensors, void* flat, void* stream);
int mc_unpack(mc_layout* L, const void* flat, void* const* tensors, void* stream);

/* mc_pack for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same copies, same validation and same errors as
 * mc_pack, but the call needs no prepared layout and performs no hipMalloc, hipFree, host-device
 * copy or synchronisation: the two small lookup tables that the gather kernel reads are rebuilt on
 * `stream`, ahead of the gather, in a fixed array of about 4 MiB inside the library's device image
 * (one copy per GPU, held until the process ends; its address is looked up on the first call on each
 * device, so make one call before starting a capture).
 * Limits: at most MC_NOALLOC_MAX_TENSORS tensors and MC_NOALLOC_MAX_ELEMS elements in total;
 * beyond either the call returns MC_ERR_LIMIT and touches nothing.
 * Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU (different
 * streams, or several host threads) race on it and must be serialised by the caller; calls queued
 * on one stream are safe. */
#define MC_NOALLOC_MAX_TENSORS 256
#define MC_NOALLOC_MAX_ELEMS (1 << 28)
int mc_pack_noalloc(const mc_layout* L, const void* const* tensors, void* flat, void* stream);

/* ---- a3 + a4: per-colour reduction fused with the SGD update -------------------------
 * Section 3, Algorithm 1 (intra-node sum, inter-node sum, then SGD on each GPU) and
 * Section 4.2 (each colour summed separately; summing ranks add the children's buffers to
 * the local GPU contributions).  For every colour c and every flat element i of colour c:
 *
 *     g    = x[o(c,0)][i]                          (start from the first term, not from 0)
 *     g    = g + x[o(c,q)][i]      for q = 1..P-1  (strictly left to right)
 *     d    = g + wd * w[i]
 *     v[i] = mu * v[i] + d
 *     w[i] = w[i] - lr * v[i]                      (uses the NEW v)
 *     grad_out[i] = g                              (if grad_out != NULL)
 *
 * every operation rounded once to fp32.  The paper gives no update formula (only that SGD is performed);
 * this is heavy-ball momentum with L2 decay folded into the gradient, dampening 0.
 *
 * contrib:  host array of P device pointers, each N fp32 flat, 16-byte aligned.  By
 *           convention entries 0..m-1 are the node's own GPU replicas and m..P-1 the tree
 *           children, so the identity sequence is Algorithm 1's order of summation.
 * order:    host, k_colours*P int32 row-major; row c is the sequence o(c,.) and must be a
 *           permutation of 0..P-1.  NULL = identity for every colour.
 * grad_out: device N fp32 or NULL; weights, momentum: device N fp32, updated in place.
 * Errors: MC_ERR_INVALID_ARG (NULL, P < 1, P > MC_MAX_P, bad order row), MC_ERR_ALIGN,
 * MC_ERR_OVERLAP (grad_out, weights or momentum overlaps another buffer of the call; the
 * contributions are only read, so the same buffer may be given twice), MC_ERR_HIP. */
int mc_reduce_update(const mc_layout* L, const void* const* contrib, int32_t P,
                     const int32_t* order, void* grad_out, void* weights, void* momentum,
                     float lr, float mu, float wd, void* stream);

/* ---- roles: the multi-colour trees and per-colour term counts -------------------------
 * Section 4.2: for each of the k colours the nodes are arranged in a k-ary breadth-first
 * spanning tree; the non-leaf nodes (root included) of different colours are disjoint; roots
 * and non-leaf nodes sum, leaves only send; the result is broadcast from the k roots.  The
 * paper's example (Figure 2): 8 nodes, 4 colours -> colour 0 rooted at node 0 with node 1 its
 * only other non-leaf, colour 1 rooted at node 2 with node 3.
 *
 * Node placement (the paper leaves it open): a tree needs s = ceil((n_nodes-1)/k) non-leaf
 * nodes; colour c fills a complete k-ary tree breadth first with the node sequence
 * c*s, c*s+1, ... (mod n_nodes).  Disjoint non-leaf sets exist iff k*s <= n_nodes; otherwise
 * both functions return MC_ERR_INVALID_ARG.  Host-only.
 *
 * mc_colour_trees: parent (host, k_colours*n_nodes int32): parent[c*n_nodes + r] is the parent
 *   of node r in colour c's tree, -1 for the root.
 * mc_rank_roles: for one rank, per colour c: role[c] (MC_ROLE_*), n_children[c], and
 *   children[c*k_colours + j] = j-th child (in arrival order), -1 beyond n_children[c]. */
enum { MC_ROLE_LEAF = 0, MC_ROLE_INNER = 1, MC_ROLE_ROOT = 2 };
int mc_colour_trees(int32_t n_nodes, int32_t k_colours, int32_t* parent);
int mc_rank_roles(int32_t n_nodes, int32_t k_colours, int32_t rank, int32_t* role,
                  int32_t* n_children, int32_t* children);

/* mc_reduce_update with a role per colour.  A rank is root or inner node of at most one
 * colour and a leaf of the others (Section 4.2), so what it adds differs by colour: as a leaf
 * only its own m GPU replicas, as inner node or root those plus one buffer per child; and only
 * the root holds the complete sum, so only there can the SGD step follow at once -- the other
 * colours' partial sums go to grad_out (to be pulled by the parent), and their update is a
 * later call with the broadcast result as the single contribution.
 *
 * n_terms:   host, k_colours int32: colour c adds the first n_terms[c] entries of its sequence
 *            (row c of order, or 0,1,2,.. if order is NULL); 0 <= n_terms[c] <= P; 0 = the
 *            colour is skipped and nothing in its range is read or written.
 * do_update: host, k_colours bytes: non-zero = apply the update for colour c (needs weights and
 *            momentum); zero = only write the sum to grad_out (needs grad_out).
 * Other arguments, arithmetic and errors as mc_reduce_update; weights / momentum may be NULL
 * when no colour updates, grad_out may be NULL when every non-skipped colour updates. */
int mc_reduce_update_roles(const mc_layout* L, const void* const* contrib, int32_t P,
                           const int32_t* order, const int32_t* n_terms, const uint8_t* do_update,
                           void* grad_out, void* weights, void* momentum,
                           float lr, float mu, float wd, void* stream);

/* ---- packets: the reduction restricted to a sub-range of the payload -------------------
 * Section 4.2: the k reductions are pipelined -- network packets of every colour move
 * concurrently and a summing rank adds each packet as it arrives rather than waiting for whole
 * chunks.  The per-packet operation is mc_reduce_update (or its roles form) restricted to the
 * flat elements [elem_begin, elem_end): every colour is cut to that range, everything outside is
 * neither read nor written.  Because the step is elementwise, running any partition of [0, N)
 * into packets, in any order and on any streams, gives bit for bit the result of the whole call.
 * The caller sequences packets against their arrival (e.g. an event wait on `stream` before
 * the call).
 *
 * elem_begin, elem_end: 0 <= begin <= end <= N, begin a multiple of MC_COLOUR_ALIGN_ELEMS, end a
 *   multiple of it or equal to N; otherwise MC_ERR_INVALID_ARG.  An empty range is a no-op.
 * n_terms, do_update: both NULL (every colour adds all P terms and updates) or both given, as in
 *   mc_reduce_update_roles.  Everything else as mc_reduce_update. */
int mc_reduce_update_range(const mc_layout* L, const void* const* contrib, int32_t P,
                           const int32_t* order, const int32_t* n_terms, const uint8_t* do_update,
                           void* grad_out, void* weights, void* momentum,
                           float lr, float mu, float wd,
                           int64_t elem_begin, int64_t elem_end, void* stream);

/* ---- fused step: no staging of the contributions, no separate unpack --------------------
 * Section 4.2's summing ranks add what arrived directly to "the local contributions from the
 * GPUs"; nothing in the method requires a copy of each contribution into a flat buffer first.
 * mc_fused_step computes exactly what  P x mc_pack + mc_reduce_update + mc_unpack  compute --
 * same flat index space, same colour chunks, same per-colour sequence, same rounding -- but
 * reads the contributions from their per-layer tensors, updates per-layer weights and momentum
 * in place, and writes the reduced gradient as the flat payload.
 *
 * A tensor set is the device-resident list of one tensor pointer per layer of a layout
 * (gradient tensors of one contribution, or the weights, or the momentum buffers).  Frameworks
 * keep these tensors at fixed addresses, so a set is created once and reused every step.
 *
 * mc_tensor_set_create: tensors = host array of n_tensors device pointers (4-byte aligned;
 *   entries of zero-length tensors are ignored).  Tensors of one set must not overlap each
 *   other.  Uploads the list (one small allocation, one synchronous copy) and prepares the
 *   layout on the current device.  The set refers to L: destroy it before L.
 *   Errors: MC_ERR_INVALID_ARG, MC_ERR_ALIGN, MC_ERR_OVERLAP, MC_ERR_ALLOC, MC_ERR_HIP.
 * mc_tensor_set_destroy: NULL is a no-op.
 *
 * mc_fused_step: contrib = host array of P sets (the same set may appear twice); order,
 *   lr, mu, wd, stream and the arithmetic as in mc_reduce_update; grad_out = device N fp32 flat,
 *   16-byte aligned, or NULL; weights, momentum = sets updated in place.  A tile whose operands
 *   are not all 16-byte aligned relative to the payload falls back to narrower accesses, never
 *   to different arithmetic.  Errors: MC_ERR_INVALID_ARG (NULL, P out of range, bad order row,
 *   a set of another layout or device), MC_ERR_ALIGN, MC_ERR_OVERLAP (weights, momentum or
 *   grad_out overlap each other or a contribution), MC_ERR_HIP. */
typedef struct mc_tensor_set mc_tensor_set;   /* opaque */
int mc_tensor_set_create(mc_layout* L, const void* const* tensors, mc_tensor_set** out);
int mc_tensor_set_destroy(mc_tensor_set* S);
/* mc_pack / mc_unpack with the tensor pointers taken from a set: one launch whatever the number of
 * tensors (the pointer-array forms need one launch per 256 tensors).  Same copies, same errors;
 * MC_ERR_INVALID_ARG also for a set of another layout or device. */
int mc_pack_set(mc_layout* L, const mc_tensor_set* tensors, void* flat, void* stream);
int mc_unpack_set(mc_layout* L, const void* flat, const mc_tensor_set* tensors, void* stream);
int mc_fused_step(mc_layout* L, const mc_tensor_set* const* contrib, int32_t P, const int32_t* order,
                  void* grad_out, const mc_tensor_set* weights, const mc_tensor_set* momentum,
                  float lr, float mu, float wd, void* stream);

/* ---- variants of the update: run-time hyper-parameters, Nesterov, the LR schedule ---------
 * Section 5 (the experimental setup): the learning rate starts at 0.1, is ramped linearly to
 * 0.1*k*n/256 (k = batch per GPU, n = number of workers), and is divided by 10 after every 30
 * epochs of a 90-epoch run.  The rate therefore changes from step to step, while a step captured
 * into a HIP graph replays fixed kernel arguments: the `_ex` entry points can read {lr, mu, wd}
 * from device memory when the kernel runs.
 *
 * mc_update_spec: lr, mu, wd are used when hyper_dev is NULL; otherwise hyper_dev points to three
 *   device floats {lr, mu, wd} (4-byte aligned) read by the kernel.  nesterov = 0 is the update of
 *   mc_reduce_update; nesterov = 1 applies the look-ahead form  w' = w - lr*(d + mu*v')  with the
 *   same d and v' (the paper names no variant; the Torch ResNet recipe it builds on uses this
 *   one).  Any other value: MC_ERR_INVALID_ARG.
 *   state_policy and sweep change how memory is walked, never a result:
 *   state_policy (MC_STATE_*): how weights and momentum are treated in the caches.  RESIDENT keeps
 *     them cached: fastest when steps run back to back, most of all on a model whose weights +
 *     momentum fit the 256 MB memory-side cache.  STREAMING treats them like the contributions:
 *     fastest when nothing of the last step is still cached because a forward / backward pass ran in
 *     between (Section 3, Algorithm 1: the gradients are computed, then summed, then applied).  The
 *     library cannot see which case it is in; DEFAULT defers to MC_OPT_STATE_POLICY (resident).
 *   sweep (MC_SWEEP_*): the direction in which a whole-payload call walks the payload.  FORWARD /
 *     BACKWARD fix it (a caller that captures steps into graphs captures one of each and
 *     alternates them).  AUTO: calls with resident state larger than the memory-side cache
 *     alternate, using a per-layout call counter (so the direction depends on the calls made so
 *     far on that layout, from any thread); all other calls walk forward.
 *   A spec must be zero-initialised apart from the fields set (unknown values: MC_ERR_INVALID_ARG).
 * mc_reduce_update_ex: the most general form of mc_reduce_update: n_terms / do_update both NULL or
 *   both given (as in _roles), range as in _range with elem_end < 0 meaning N.
 * mc_fused_step_ex: mc_fused_step with a spec and with per-colour roles: n_terms / do_update both
 *   NULL or both given, as in mc_reduce_update_roles (weights / momentum may be NULL when no colour
 *   updates, grad_out when every non-skipped colour updates).  With flat receive buffers wrapped
 *   as tensor sets this is a rank's whole step in a tree Allreduce without any staging copy.
 * mc_hyper_write: enqueues on `stream` a write of {lr, mu, wd} to hyper_dev (a one-thread kernel;
 *   no host memory is read after the call returns, nothing synchronises). */
enum { MC_STATE_DEFAULT = 0, MC_STATE_RESIDENT = 1, MC_STATE_STREAMING = 2 };
enum { MC_SWEEP_AUTO = 0, MC_SWEEP_FORWARD = 1, MC_SWEEP_BACKWARD = 2 };
typedef struct mc_update_spec {
    float lr, mu, wd;
    const float* hyper_dev;
    int32_t nesterov;
    int32_t state_policy;
    int32_t sweep;
} mc_update_spec;
int mc_reduce_update_ex(const mc_layout* L, const void* const* contrib, int32_t P,
                        const int32_t* order, const int32_t* n_terms, const uint8_t* do_update,
                        void* grad_out, void* weights, void* momentum, const mc_update_spec* spec,
                        int64_t elem_begin, int64_t elem_end, void* stream);
int mc_fused_step_ex(mc_layout* L, const mc_tensor_set* const* contrib, int32_t P, const int32_t* order,
                     const int32_t* n_terms, const uint8_t* do_update, void* grad_out,
                     const mc_tensor_set* weights, const mc_tensor_set* momentum,
                     const mc_update_spec* spec, void* stream);
int mc_hyper_write(float* hyper_dev, float lr, float mu, float wd, void* stream);

/* ---- packets consumed as they arrive: the pipelined reduction ------------------------------
 * Section 4.2: the k reductions are pipelined, packets of all colours are in flight at once and a
 * summing rank adds each packet when it has arrived.  mc_reduce_update_range leaves the sequencing
 * to the caller (an event wait per packet, tens of microseconds each on this platform);
 * mc_reduce_update_packets moves it into ONE resident kernel: its workgroups walk the packets in
 * their order of arrival and, before touching packet j, poll the device-memory flag ready[j] until it
 * equals arrivals x (the packet's length in elements): the flag counts the elements that have landed,
 * `arrivals` being the number of contributions that arrive per packet.  Whatever delivers a packet --
 * a copy kernel, a peer GPU, a network adapter -- writes the data into the contribution buffer
 * first and then raises the flag with release semantics at device scope.  Two ways are provided:
 * mc_packet_deliver copies n_elems fp32 from src to dst (device, 16-byte aligned, not overlapping)
 * and then, from a second launch behind the copy, adds n_elems to *flag once (a writer should touch
 * the polled word once per delivery: an add per workgroup of the copy serialises on it and is
 * slowed further by every poller);  mc_packet_signal stores a
 * value into ready[packet] from a kernel on `stream`, i.e. after everything queued there before it.
 *
 * Every wait is bounded: a workgroup polls at most spin_limit times in total (half a microsecond to
 * four microseconds apart, backing off while it waits) and then stops; no packet is ever left
 * half-summed.  progress (device, n_blocks + MC_PACKETS_STATUS_WORDS uint32) records per workgroup how many packets it has completed; a later
 * call with the same packets, flags, progress and n_blocks resumes every workgroup from its own
 * count.  The protocol of one step:
 *   mc_packets_reset(ready, n_packets, progress, n_blocks, stream)         -- zero both
 *   mc_reduce_update_packets(...) on the compute stream, while the producer signals packets
 *   make the compute stream wait for the producer's last signal (an event), then call
 *   mc_reduce_update_packets(...) once more with the same arguments: it finds every flag set and
 *   finishes whatever the first call gave up on (nothing, if that call saw all packets).
 * After that call progress[b] == n_packets for every b < n_blocks, progress[n_blocks] counts the
 * workgroups that ever stopped waiting, and progress[n_blocks + 1] is non-zero if a packet descriptor
 * was not a range inside one colour (such packets are skipped).
 *
 * packets: device, 2 * n_packets int64: begin and end of each packet in arrival order; each must be
 *   a range as mc_reduce_update_range requires and lie inside one colour; the packets of a step
 *   must be disjoint and should cover the payload.  (Device arrays cannot be validated on the host.)
 * ready: device, n_packets uint32.  arrivals: >= 1.  n_blocks: workgroups of 256 threads, at least 1
 *   and at most twice the device's compute units (MC_ERR_LIMIT beyond: all workgroups have to be
 *   resident together and still leave wave slots to the kernels that deliver packets, or each side
 *   waits for the other until the poll budget ends).  One per compute unit is a good choice.
 * Every colour adds all P terms and updates (order, spec, grad_out as in mc_reduce_update_ex).
 * Limits: at most MC_PACKETS_MAX_COLOURS colours and k_colours * P <= 256 (MC_ERR_LIMIT).
 * Errors otherwise as mc_reduce_update_ex. */
#define MC_PACKETS_MAX_COLOURS 32
#define MC_PACKETS_MAX_BLOCKS 4096
#define MC_PACKETS_STATUS_WORDS 2
int mc_packets_reset(uint32_t* ready, int32_t n_packets, uint32_t* progress, int32_t n_blocks, void* stream);
int mc_packet_signal(uint32_t* ready, int32_t packet, uint32_t value, void* stream);
int mc_packet_deliver(void* dst, const void* src, int64_t n_elems, uint32_t* flag, void* stream);
int mc_reduce_update_packets(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
                             void* grad_out, void* weights, void* momentum, const mc_update_spec* spec,
                             const int64_t* packets, int32_t n_packets, const uint32_t* ready,
                             uint32_t arrivals, uint32_t spin_limit, uint32_t* progress, int32_t n_blocks,
                             void* stream);

/* The schedule of Section 5 as a function of the position in training, in epochs (fractions
 * allowed): with target = base_lr * batch_per_gpu * n_workers / 256,
 *   epoch <  warmup_epochs:  base_lr + (target - base_lr) * epoch / warmup_epochs
 *   epoch >= warmup_epochs:  target / 10^floor(epoch / drop_every_epochs)
 * The paper gives base_lr = 0.1, drop_every_epochs = 30 and a 90-epoch run; it does not say how
 * long the ramp lasts (the schedule it cites ramps over 5 epochs), so that is an argument.
 * Host-only.  Writes the rate to *lr_out.  Errors: MC_ERR_INVALID_ARG (NULL, base_lr not finite
 * or <= 0, batch_per_gpu < 1, n_workers < 1, warmup_epochs < 0, drop_every_epochs <= 0,
 * epoch < 0 or not finite). */
int mc_lr_schedule(float base_lr, int32_t batch_per_gpu, int32_t n_workers, float warmup_epochs,
                   float drop_every_epochs, float epoch, float* lr_out);

/* ---- diagnostics and tuning ---------------------------------------------------------- */
/* Plain device-to-device copy of n_bytes (a multiple of 16; dst and src device, 16-byte
 * aligned, not overlapping) with the library's own 128-bit streaming kernel.  Not part of the
 * method: it is the yardstick for achievable HBM bandwidth and the known-size traffic that
 * hardware counters are calibrated against.  Errors: MC_ERR_INVALID_ARG, MC_ERR_ALIGN,
 * MC_ERR_OVERLAP, MC_ERR_HIP. */
int mc_copy(void* dst, const void* src, int64_t n_bytes, void* stream);
/* Occupies one wavefront on `stream` for about `microseconds` (at most 100000; bounded in the kernel
 * as well): the stand-in, in measurements, for the time a packet spends on a wire.  Not part of
 * the method. */
int mc_delay(uint32_t microseconds, void* stream);

const char* mc_strerror(int code);     /* static string, never NULL */
int mc_last_hip_error(void);           /* raw hipError_t of this thread's last MC_ERR_HIP */

/* Launch-shape knobs for measurement sweeps; results never depend on them.
 * Returns MC_ERR_INVALID_ARG for an unknown option or a value outside its range. */
enum {
    MC_OPT_RU_SHAPE = 1,           /* workgroup shape of reduce_update and fused_step: 1 = 64 threads x
                                      one 16-byte vector, 2 = 256 threads x two vectors; 0 (default) =
                                      the library's choice (the one-wavefront shape: it measured
                                      fastest or level on every configuration) */
    MC_OPT_STATE_POLICY = 2,       /* what MC_STATE_DEFAULT means: MC_STATE_RESIDENT (default) or
                                      MC_STATE_STREAMING */
    MC_OPT_PACK_NONTEMPORAL = 3,   /* pack/unpack: bit 0 streaming access to the per-layer
                                      tensors, bit 1 streaming access to the flat payload
                                      (non-temporal loads, write-through stores) */
    MC_OPT_STATE_STORE_SC1 = 4,    /* 0 / 1: resident-policy tiles store updated weights and momentum
                                      with the agent-scope (write-through) bit */
    MC_OPT_ALTERNATE_SWEEP = 5,    /* 0 / 1: whether MC_SWEEP_AUTO alternates at all */
    MC_OPT_XCD_RUN = 6,            /* 0..64: workgroups are dealt to the chip's 8 dies round-robin;
                                      with a value r > 1 the reduce_update and fused_step kernels
                                      permute their tiles so that each die walks r consecutive tiles
                                      (neighbouring tiles then share one L2).  0 or 1: tile =
                                      workgroup index. */
    MC_OPT_XCD_RUN_PACK = 7,       /* the same for mc_pack / mc_pack_set; -1 (default) = chosen from the
                                      payload size */
    MC_OPT_XCD_RUN_UNPACK = 8,     /* the same for mc_unpack / mc_unpack_set */
    MC_OPT_DIRECT_TILES = 9,       /* how a workgroup finds its work.  1 (default): reduce_update divides
                                      the tile index by the chunk length to get the colour, fused_step
                                      walks the layout's tensor-aligned units (mc_layout_units);
                                      2: fused_step uses flat 256-element tiles like reduce_update;
                                      0: both search a per-launch table of colour segments */
    MC_OPT_LDS_CAP_UPDATE = 10,    /* bytes of unused LDS reserved per workgroup of reduce_update and
                                      fused_step (0..65536), which caps the workgroups resident per
                                      compute unit and so the number of loads in flight; -1 (default)
                                      = by the call: none while weights and momentum are expected in
                                      the memory-side cache, otherwise as many wavefronts per compute
                                      unit as keep about 80 KB of loads in flight (14 for four
                                      contributions, 8 for eight); 0 = no cap */
    MC_OPT_LDS_CAP_PACK = 11       /* the same for pack, unpack and mc_copy; default 0 (no cap) */
};
int mc_set_option(int option, int value);
int mc_get_option(int option, int* value);

#ifdef __cplusplus
}
#endif
#endif /* MC_H_ */
