/*
 * ddlsync.h -- C ABI of the MI355X (gfx950) synchronizer hot path of Decoupled DiLoCo.
 *
 * What the library computes, for one fragment p of the model (Algorithm 2, steps "Weight",
 * "mergeFn" and "OuterOpt"; Appendix D.2 "Direct averaging", weighted form; Section 2 for
 * the outer optimiser):
 *
 *     r_m     = q_m * n_m                       raw weight: token counter of learner m if it
 *                                               is in the reporting set M_t, else 0
 *     w_m     = r_m / sum_k r_k                 normalised over the quorum
 *     Delta_i = sum_m w_m (Theta_i - theta_{m,i})      outer gradient, old global minus learner
 *     v_i     <- mu v_i + Delta_i                       SGD with Nesterov momentum,
 *     Theta_i <- Theta_i - lr (Delta_i + mu v_i)        buffer form, v_i being the new buffer
 *
 * Theta (the global fragment) and v (its momentum buffer) are fp32 arrays in device memory
 * and are updated in place by one fused pass; learner fragments are bf16 or fp32 device
 * arrays that are read exactly once, and only if the learner contributes (q_m = 1 and
 * n_m > 0).  A learner that does not contribute is never dereferenced: its pointer may be
 * NULL, dangling, or point at NaNs (Section 4, "Syncer worker": an absent learner takes part
 * in the same Merge with weight 0).
 *
 * Conventions common to all entry points
 *   - "host" / "device" in a parameter comment says where the memory lives.  The caller owns
 *     every buffer.  Host arrays are read before the call returns; device buffers must stay
 *     valid until the stream has run the enqueued work.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and return; they do not wait for the GPU.
 *   - Argument errors are detected before anything is enqueued: on any status other than
 *     DDL_OK, Theta and v of every fragment in the call are untouched.
 *   - Theta and v need 4-byte alignment, learner arrays the natural alignment of their
 *     element.  Arrays whose base addresses are all 16-byte aligned take 128-bit vector
 *     accesses; anything else is handled by an element-wise path with the same results.
 *   - Theta and v ranges must not overlap each other nor any contributing learner range
 *     (DDL_ERR_ALIAS); learner ranges may overlap one another.
 *   - Entry points may be called from several host threads; calls that touch the same Theta
 *     or v must be ordered by the caller (same stream, or events).  No launch path takes a
 *     lock.
 *   - Process-wide state, all of it: (1) the launch-shape options of ddl_set_option, atomics
 *     that every later call on any thread reads -- a measurement aid, results never depend on
 *     them; (2) the staging cache of ddl_merge_batch (per device, up to 64 descriptor tables in
 *     library-owned pinned-host and device buffers, behind one mutex that is held while that
 *     call enqueues, never while it waits for the GPU; freed when the process ends); (3) the
 *     fixed scratch array of ddl_rda_merge_fragment_static.  Plans hold everything else.
 *   - lr and mu must be finite and >= 0.
 */
#ifndef DDLSYNC_H
#define DDLSYNC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Entry points are the library's only exported symbols. */
#define DDL_API __attribute__((visibility("default")))

typedef enum {
    DDL_OK = 0,
    DDL_ERR_INVALID_ARG = 1,  /* NULL where data is needed, M out of range, mask not 0/1, ...  */
    DDL_ERR_EMPTY_QUORUM = 2, /* sum_k q_k n_k == 0: no merge is defined                        */
    DDL_ERR_ALIAS = 3,        /* an output range overlaps another range of the call             */
    DDL_ERR_RUNTIME = 4       /* a HIP call failed (see ddl_last_error_message)                 */
} ddl_status;

typedef enum { DDL_F32 = 0, DDL_BF16 = 1 } ddl_dtype;

/* The paper runs M in {2, 4, 8, 16} (Tables 1 and 11). */
#define DDL_MAX_LEARNERS 16

/* Library version, major * 10000 + minor * 100 + patch. */
DDL_API int ddl_version(void);

/* Static string naming the sources this library was built from: twelve hex digits of a hash
 * over the kernel and host sources and this header ("unknown" if the build did not set it).
 * Profile summaries record it next to counter figures, so that a figure taken on other
 * kernels is not mistaken for a current one. */
DDL_API const char* ddl_build_id(void);

/* The same for one kernel family -- "merge" (direct averaging), "rda", "q4": a hash over only
 * the sources that decide that family's code, so that an unrelated change elsewhere does not
 * age its counter figures.  "" for an unknown name. */
DDL_API const char* ddl_kernel_build_id(const char* kernel);

/* Static string for a status code. */
DDL_API const char* ddl_status_string(ddl_status s);

/* Text of the last DDL_ERR_RUNTIME on the calling thread ("" if none); a refusal for lack of
 * scratch space (DDL_ERR_INVALID_ARG of the RDA entry points) also leaves the sizes here.
 * Thread-local storage owned by the library, valid until the thread's next failing call. */
DDL_API const char* ddl_last_error_message(void);

/*
 * Weight, tokens-only form (Algorithm 2 "Weight"; normalisation as in the denominator of the
 * weighted merge, Appendix D.2): w_out[m] = q_m n_m / sum_k q_k n_k, in fp64.
 * token_counts, quorum_mask, w_out: host arrays of M entries.  quorum_mask entries are 0 or 1.
 * Errors: INVALID_ARG (NULL, M < 1, M > DDL_MAX_LEARNERS, mask entry > 1), EMPTY_QUORUM.
 */
DDL_API ddl_status ddl_compute_weights(const uint64_t* token_counts, const uint8_t* quorum_mask,
                                       int M, double* w_out);

/*
 * The paper's own Weight function (Section 3.2): raw weight c_tokens * (c_tokens / c_steps),
 * "quantity times quality", zero for learners outside the quorum, normalised over the quorum.
 * A quorum member with c_steps = 0 and c_tokens = 0 gets weight 0; c_steps = 0 with
 * c_tokens > 0 is INVALID_ARG.  All arrays: host, M entries.
 */
DDL_API ddl_status ddl_compute_weights_quality(const uint64_t* token_counts,
                                               const uint64_t* step_counts,
                                               const uint8_t* quorum_mask, int M, double* w_out);

/*
 * One fragment held as ONE flat array: Weight, Merge and OuterOpt as defined at the top of
 * this file (Algorithm 2, steps Weight / mergeFn / OuterOpt).
 *
 *   theta, v        device, n fp32 elements each, updated in place
 *   learner_params  HOST array of M DEVICE pointers, learner m's copy of the fragment, n
 *                   elements of learner_dtype; entries of non-contributing learners are
 *                   never dereferenced
 *   token_counts    host, M entries: tokens learner m processed since its last sync of this
 *                   fragment (Algorithm 1's c^tokens)
 *   quorum_mask     host, M entries, 1 if learner m is in the reporting set M_t
 *   n               elements; n == 0 is DDL_OK and enqueues nothing
 *
 * Everything the kernel needs travels in its argument block: no device allocation, no copy.
 */
DDL_API ddl_status ddl_merge_fragment(float* theta, float* v, const void* const* learner_params,
                                      ddl_dtype learner_dtype, const uint64_t* token_counts,
                                      const uint8_t* quorum_mask, int M, size_t n, float lr,
                                      float mu, void* hip_stream);

/*
 * As ddl_merge_fragment, with normalised weights supplied by the caller instead of token
 * counters and mask (for the quantity-times-quality Weight function or any other):
 * weights is a host array of M non-negative finite fp64 values with a positive sum; they are
 * divided by their sum in fp64 before use.  w_m == 0 marks a non-contributing learner.
 */
DDL_API ddl_status ddl_merge_fragment_weighted(float* theta, float* v,
                                               const void* const* learner_params,
                                               ddl_dtype learner_dtype, const double* weights,
                                               int M, size_t n, float lr, float mu,
                                               void* hip_stream);

/*
 * As ddl_merge_fragment, and in the same pass also writes the new Theta, rounded to
 * nearest-even bf16, into theta_bf16 (device, n bf16 elements, not NULL): the fragment as it
 * is broadcast back to the learners (Algorithm 2, "Send(Learners, Theta_p, t)"), without a
 * second sweep over Theta.  Costs 2 more bytes of HBM traffic per parameter.
 */
DDL_API ddl_status ddl_merge_fragment_bcast(float* theta, float* v, void* theta_bf16,
                                            const void* const* learner_params,
                                            ddl_dtype learner_dtype, const uint64_t* token_counts,
                                            const uint8_t* quorum_mask, int M, size_t n, float lr,
                                            float mu, void* hip_stream);

/*
 * As ddl_merge_fragment, and the same pass also writes the merged outer gradient it applied,
 *
 *     Delta_i = sum_m w_m (Theta_i - theta_{m,i})        (Appendix D.2, weighted direct averaging)
 *
 * into delta_out (device, n fp32 elements; it may overlap no other array of the call): for
 * inspecting the outer gradient -- its norm, its cosine to a learner's, a caller's own outer
 * optimiser run beside the fused one -- without another sweep over the learners' copies.
 * Theta and v come out bit for bit as from ddl_merge_fragment.  delta_out == NULL makes the
 * call ddl_merge_fragment itself.  Costs 4 more bytes of HBM traffic per parameter; no device
 * allocation, no copy.
 */
DDL_API ddl_status ddl_merge_fragment_ex(float* theta, float* v, float* delta_out,
                                         const void* const* learner_params,
                                         ddl_dtype learner_dtype, const uint64_t* token_counts,
                                         const uint8_t* quorum_mask, int M, size_t n, float lr,
                                         float mu, void* hip_stream);

/*
 * Radial-directional averaging (Appendix D.2, "Radial-directional averaging", weighted form)
 * as the merge, fused with the same outer Nesterov step, for one flat tensor.  With
 * d_m = Theta - theta_m over a group of elements and normalised weights w_m,
 *
 *     Delta = ( sum_m w_m ||d_m|| ) * phi( sum_m w_m phi(d_m) ),     phi(x) = x / ||x||_2
 *
 * so norms and directions are averaged separately (the paper merges the non-embedding
 * parameters this way, Section 5.1).  Readings where the paper is silent or garbled: the first
 * factor of the printed weighted formula is the weighted mean of the norms; one norm is taken
 * per group of `group_len` consecutive elements (group_len = row length: one magnitude per
 * row; group_len >= n: one per tensor; the last group may be shorter); a learner whose outer
 * gradient is zero on a group adds no direction there; a zero mean direction gives Delta = 0.
 *
 *   workspace        device scratch of at least ddl_rda_workspace_bytes(n, group_len, M) bytes,
 *                    256-byte aligned, owned by the caller, overwritten; it must stay valid
 *                    until the stream has run the call and must not be shared by calls that
 *                    may overlap in time
 *   other arguments  as ddl_merge_fragment
 *
 * Allocates nothing.  Many groups of at most 16384 elements on 16-byte-aligned arrays (n and
 * group_len multiples of four) take one kernel that reads every byte once; many other moderate
 * groups take one kernel that sweeps each group three times, the later sweeps served from the
 * caches; long or few groups take three kernels that read the learners and Theta twice (a sweep
 * for the Gram matrix of the outer gradients, a per-group reduction, the outer step) -- five
 * kernels and three reads with more than eleven contributing learners.  Results are
 * reproducible (no atomics).
 * Errors as ddl_merge_fragment, plus INVALID_ARG for group_len == 0 or a workspace that is
 * NULL, misaligned or too small, and ALIAS if the workspace overlaps any array of the call.
 */
DDL_API size_t ddl_rda_workspace_bytes(size_t n, size_t group_len, int M);
DDL_API ddl_status ddl_rda_merge_fragment(float* theta, float* v, const void* const* learner_params,
                                          ddl_dtype learner_dtype, const uint64_t* token_counts,
                                          const uint8_t* quorum_mask, int M, size_t n,
                                          size_t group_len, float lr, float mu, void* workspace,
                                          size_t workspace_bytes, void* hip_stream);

/*
 * ddl_rda_merge_fragment for callers that cannot allocate device memory and have no workspace
 * to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same kernels, same results; the scratch
 * is a fixed array of ddl_rda_static_scratch_bytes() = 4 MiB inside the library's device
 * image, which every GPU the library runs on holds until the process ends.  The call
 * allocates nothing on the device (no hipMalloc, no hipFree, no allocating library routine);
 * its first call on a device looks the array's address up.
 *
 * A tensor and grouping that need more scratch than that -- ddl_rda_workspace_bytes(n,
 * group_len, M) above 4 MiB, which takes about 10^8 elements in one group at sixteen learners
 * (more with fewer) or about 10^5 groups -- are refused with DDL_ERR_INVALID_ARG before anything is
 * enqueued (ddl_last_error_message gives the sizes); use the workspace form for those.
 * All calls on one GPU share the one array and it keeps the last call's contents; nothing in
 * it has to start at zero (every kernel writes what it later reads).  Calls that may overlap
 * in time on one GPU (different streams, different threads) race on it: keep them on one
 * stream or order them with events.
 */
DDL_API size_t ddl_rda_static_scratch_bytes(void);
DDL_API ddl_status ddl_rda_merge_fragment_static(float* theta, float* v,
                                                 const void* const* learner_params,
                                                 ddl_dtype learner_dtype,
                                                 const uint64_t* token_counts,
                                                 const uint8_t* quorum_mask, int M, size_t n,
                                                 size_t group_len, float lr, float mu,
                                                 void* hip_stream);

/*
 * 4-bit outer gradients (Appendix D.3, "Outer gradients compression": outer gradients are
 * compressed from bf16 to int4 before the merge).  The paper fixes only the width; the format
 * is this library's, a plain symmetric block-wise integer quantiser:
 *   - the flat fragment is cut into blocks of block_len consecutive elements (block_len a
 *     multiple of 8, at least 8; the last block may be shorter);
 *   - per learner, block b has one fp32 scale and element i a signed 4-bit code in two's
 *     complement, two codes per byte: element 2k in the low nibble of byte k, element 2k + 1 in
 *     its high nibble; (n + 1) / 2 bytes of codes, ceil(n / block_len) scales;
 *   - a (scale, code) pair stands for the outer-gradient value scale * code.
 *
 * ddl_q4_encode        the learner side: d = Theta - theta_m in fp32, scale = max|d| / 7 over
 *                      the block, code = round-half-even(d / scale) clamped to [-7, 7]; a block
 *                      of zeros gets scale 0 and codes 0.  theta, learner_params: device, n
 *                      elements, 16-byte aligned; codes_out, scales_out: device, 4-byte aligned,
 *                      written (an unused high nibble is 0).  Reproducible bit for bit.
 * ddl_q4_merge_fragment   the syncer side: Delta_i = sum_m w_m scale_m[i / block_len] code_m[i]
 *                      with the quorum weights of ddl_merge_fragment, then the same outer
 *                      Nesterov step, in place on theta and v (device, 16-byte aligned).
 *                      codes, scales: HOST arrays of M DEVICE pointers (4-byte aligned); entries
 *                      of learners of weight zero are never read and may be NULL.
 * Both only enqueue a kernel.  Errors as ddl_merge_fragment; INVALID_ARG also for a bad
 * block_len or a misaligned array, ALIAS if an output overlaps any other array of the call.
 */
DDL_API ddl_status ddl_q4_encode(const float* theta, const void* learner_params,
                                 ddl_dtype learner_dtype, size_t n, size_t block_len,
                                 uint8_t* codes_out, float* scales_out, void* hip_stream);
DDL_API ddl_status ddl_q4_merge_fragment(float* theta, float* v, const uint8_t* const* codes,
                                         const float* const* scales, const uint64_t* token_counts,
                                         const uint8_t* quorum_mask, int M, size_t n,
                                         size_t block_len, float lr, float mu, void* hip_stream);

/*
 * A fragment as the paper forms it: a set of whole tensors (Section 5.1 and Appendix C,
 * balanced tensor fragmentation), each tensor its own flat array ("segment").  All segments of
 * a fragment share the fragment's counters, mask, lr and mu (per-fragment counters c_{m,p},
 * Section 3.1).
 */
typedef struct ddl_segment {
    float* theta;                      /* device, n fp32 elements, updated in place            */
    float* v;                          /* device, n fp32 elements, updated in place            */
    const void* const* learner_params; /* HOST array of M DEVICE pointers (M of the fragment)  */
    size_t n;                          /* elements in this tensor; 0 is allowed                */
    void* theta_bf16;                  /* device, optional (NULL: none): n bf16 elements that
                                          receive the new Theta rounded to nearest-even, the
                                          copy the syncer sends back to the learners
                                          (Algorithm 2, "Send(Learners, Theta_p)"), written by
                                          the same pass; 2-byte aligned, must overlap nothing  */
} ddl_segment;

typedef struct ddl_fragment {
    const ddl_segment* segs;      /* host array of num_segs segments                           */
    int num_segs;                 /* >= 0                                                      */
    ddl_dtype learner_dtype;      /* element type of every learner array of this fragment     */
    const uint64_t* token_counts; /* host, M entries                                           */
    const uint8_t* quorum_mask;   /* host, M entries of 0/1                                    */
    int M;                        /* 1 .. DDL_MAX_LEARNERS                                     */
    float lr, mu;                 /* outer learning rate and momentum of this fragment         */
} ddl_fragment;

/*
 * Batched streaming variant: merge num_frags fragments, each made of several tensors and each
 * with its own quorum, counters, lr and mu, as one piece of enqueued work (Section 5.1: one
 * fragment is synchronised per training step and two are in flight; small tensors such as MoE
 * experts and routers must still fill the GPU).  Equivalent to calling ddl_merge_fragment on
 * every segment of every fragment; fragments of one call must be distinct (no Theta or v
 * range may appear twice: DDL_ERR_ALIAS).
 *
 * The segment descriptors are staged through library-owned, lazily grown pinned-host and
 * device buffers, and the last 64 distinct tables stay there: a call that names the same
 * fragments (same pointers and sizes) as an earlier one reuses its table without any copy.
 * A call may allocate (new table, or growth) and may wait for an earlier call that still uses
 * the buffer it takes over.  Not capturable in a HIP graph: on a stream that is being captured
 * the call returns DDL_ERR_INVALID_ARG and enqueues nothing (use a plan for that).
 */
DDL_API ddl_status ddl_merge_batch(const ddl_fragment* frags, int num_frags, void* hip_stream);

/*
 * Resident plan: the same batched merge for a syncer whose buffers persist across syncs
 * (Section 4, "Syncer worker": the syncer keeps the global parameters and the outer optimiser
 * state, and one shard per learner persists even while the learner is away).  The segment
 * descriptors of ALL fragments of the model are built and uploaded once; each sync then only
 * passes the per-sync inputs of the fragments that are due, and enqueues kernels with no
 * allocation and no copy.
 *
 * ddl_plan_create reads frags[i].segs / num_segs / learner_dtype / M; token_counts,
 * quorum_mask, lr and mu of the fragments are ignored there (may be NULL / 0).  Every learner
 * pointer must be valid device memory or NULL.  The plan is bound to the device that is
 * current at creation.  *plan_out is NULL on error.
 */
typedef struct ddl_plan ddl_plan;

typedef struct ddl_sync {
    int fragment;                 /* index into the plan's fragments                           */
    const uint64_t* token_counts; /* host, M entries (M of that fragment)                      */
    const uint8_t* quorum_mask;   /* host, M entries of 0/1                                    */
    float lr, mu;
} ddl_sync;

DDL_API ddl_status ddl_plan_create(const ddl_fragment* frags, int num_frags, ddl_plan** plan_out);

/* Merge the fragments named by syncs[0..count) (distinct fragment indices). A contributing
 * learner whose pointer was NULL at plan creation is INVALID_ARG. */
DDL_API ddl_status ddl_plan_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                  void* hip_stream);

/* Frees the plan's device table. The caller must first make sure no enqueued merge of this
 * plan is still running. NULL is a no-op. */
DDL_API ddl_status ddl_plan_destroy(ddl_plan* plan);

/* Number of fragments / total elements of a plan (0 for NULL). */
DDL_API int ddl_plan_num_fragments(const ddl_plan* plan);
DDL_API size_t ddl_plan_num_elements(const ddl_plan* plan);

/*
 * Radial-directional averaging (Appendix D.2; see ddl_rda_merge_fragment for the formula and
 * the readings) through a plan: the fragments named by the syncs are merged tensor by tensor,
 * each tensor in groups of its own length, and all tensors of a fragment whose groups fit the
 * one-pass kernel go out in ONE launch per group-length class (up to 1024, 1536, 2048, 4096,
 * 8192, 16384 elements) instead of one launch per tensor.
 *
 * ddl_plan_set_rda_groups   group_len[s] for every segment the plan was created with, empty
 *                           ones included, fragment by fragment in creation order
 *                           (num_segments = their total); 0 or a value above the segment's n
 *                           means one group for the whole tensor; (size_t)-1 means that this
 *                           tensor is merged by direct averaging, not RDA (the paper uses RDA
 *                           for the non-embedding parameters only, Section 5.1).  Uploads a small device
 *                           table (allocates; not for capture); may be called again to change
 *                           the grouping once no merge of the plan is running.
 * ddl_plan_rda_workspace_bytes   size of the scratch the merges of this plan need (0 before
 *                           ddl_plan_set_rda_groups): the largest ddl_rda_workspace_bytes over
 *                           the plan's tensors.
 * ddl_plan_rda_merge        as ddl_plan_merge, with the RDA merge.  workspace: device scratch,
 *                           256-byte aligned, at least ddl_plan_rda_workspace_bytes(plan),
 *                           overwritten, not shared by calls that may overlap in time.  Only
 *                           enqueues kernels.  A segment's optional theta_bf16 receives the
 *                           new Theta as bf16 in the same pass, as in ddl_plan_merge.
 * Errors as ddl_plan_merge; INVALID_ARG also if the groups were never set, num_segments does
 * not match the plan, or the workspace is NULL, misaligned or too small; ALIAS if the
 * workspace overlaps an array of a fragment that is due.  Theta and v are untouched on error.
 */
DDL_API ddl_status ddl_plan_set_rda_groups(ddl_plan* plan, const size_t* group_len,
                                           size_t num_segments);
DDL_API size_t ddl_plan_rda_workspace_bytes(const ddl_plan* plan);
DDL_API ddl_status ddl_plan_rda_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * 4-bit outer gradients (Appendix D.3; format as defined at ddl_q4_encode) through a plan: the
 * fragments named by the syncs are merged from the learners' codes and scales instead of their
 * parameter copies, whole fragments of many tensors per kernel launch, exactly as
 * ddl_plan_merge does for bf16 / fp32 learners.  Each tensor of a learner is encoded on its own
 * (blocks never straddle tensors), as ddl_q4_encode writes it.
 *
 * ddl_plan_set_q4_sources   segs[s] for every segment the plan was created with, empty ones
 *                           included, fragment by fragment in creation order (num_segments =
 *                           their total): HOST arrays of M DEVICE pointers to learner m's
 *                           codes ((n + 1) / 2 bytes) and scales (ceil(n / block_len) floats) of
 *                           that tensor, 4-byte aligned; both NULL for a learner that will never
 *                           contribute there.  The plan's learner pointers are not used by the
 *                           4-bit merge and may have been NULL at creation.  Theta and v of every
 *                           non-empty tensor must be 16-byte aligned (a theta_bf16, 8-byte).
 *                           Uploads a device table (allocates; not for capture); may be called
 *                           again once no merge of the plan is running.
 * ddl_plan_q4_merge         as ddl_plan_merge.  Only enqueues kernels; a segment's optional
 *                           theta_bf16 receives the new Theta as bf16 in the same pass.
 * Errors as ddl_plan_merge; INVALID_ARG also if the sources were never set, num_segments does
 * not match, block_len is bad, an array is misaligned, or a contributing learner has no
 * sources in some tensor of a fragment that is due; ALIAS if a source array overlaps Theta, v
 * or a bf16 copy of the plan.  Theta and v are untouched on error.
 */
typedef struct ddl_q4_segment {
    const uint8_t* const* codes; /* HOST array of M DEVICE pointers (M of the fragment)         */
    const float* const* scales;  /* HOST array of M DEVICE pointers                              */
} ddl_q4_segment;

DDL_API ddl_status ddl_plan_set_q4_sources(ddl_plan* plan, const ddl_q4_segment* segs,
                                           size_t num_segments, size_t block_len);
DDL_API ddl_status ddl_plan_q4_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                     void* hip_stream);

/*
 * Radial-directional averaging as the merge of 4-bit outer gradients: what the syncer runs
 * when the outer gradients arrive compressed (Appendix D.3: they are compressed before the
 * mergeFn of Algorithm 2) and the mergeFn is RDA (Appendix D.2; Section 5.1).  The outer
 * gradient of learner m at element i is scale_m[i / block_len] * code_m[i]; norms are taken
 * over groups of group_len consecutive elements of a tensor (groups and scale blocks need not
 * line up), Delta is the RDA formula given at ddl_rda_merge_fragment, then the same outer
 * Nesterov step.  Same kernels as the RDA merge of bf16 / fp32 learners, instantiated for codes
 * and scales (the reducing sweeps then read neither Theta nor v).
 *
 * ddl_q4_rda_merge_fragment   one tensor: arguments of ddl_q4_merge_fragment plus group_len and
 *                             the workspace of ddl_rda_merge_fragment
 *                             (ddl_rda_workspace_bytes(n, group_len, M) bytes).
 * ddl_plan_q4_rda_merge       whole fragments through a plan on which both
 *                             ddl_plan_set_q4_sources and ddl_plan_set_rda_groups have been
 *                             called; arguments and workspace as ddl_plan_rda_merge.  A tensor
 *                             whose group length is (size_t)-1 takes the direct 4-bit merge.
 * Both only enqueue kernels.  Errors as ddl_q4_merge_fragment / ddl_plan_rda_merge.
 */
DDL_API ddl_status ddl_q4_rda_merge_fragment(float* theta, float* v, const uint8_t* const* codes,
                                             const float* const* scales,
                                             const uint64_t* token_counts,
                                             const uint8_t* quorum_mask, int M, size_t n,
                                             size_t block_len, size_t group_len, float lr,
                                             float mu, void* workspace, size_t workspace_bytes,
                                             void* hip_stream);
DDL_API ddl_status ddl_plan_q4_rda_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                         void* workspace, size_t workspace_bytes,
                                         void* hip_stream);

/*
 * Balanced tensor fragmentation (Section 5.1; Appendix C, "Balanced tensor fragmentation"):
 * greedy number partitioning of the model's tensors into num_fragments fragments -- tensors are
 * taken in descending order of size and each goes to the fragment whose total is the smallest
 * so far (largest fragment at most 4/3 of the optimum).  Ties, on which the paper is silent:
 * equal sizes keep their input order; the lowest-numbered of equally light fragments wins.
 *   sizes        host, num_tensors entries, any unit (elements, bytes, bits)
 *   fragment_of  host, num_tensors entries, receives the fragment index of each tensor
 * Host-only; produces the tensor lists that ddl_plan_create / ddl_merge_batch take.
 * Errors: INVALID_ARG (num_tensors < 0, num_fragments < 1, NULL with num_tensors > 0).
 */
DDL_API ddl_status ddl_balanced_fragments(const uint64_t* sizes, int num_tensors, int num_fragments,
                                          int* fragment_of);

/*
 * Measurement aid, not part of the method: a plain device-to-device streaming copy of `bytes`
 * bytes (a multiple of 16; dst and src device, 16-byte aligned, not overlapping) with the
 * merge kernel's access width and cache hints.  It reads `bytes` and writes `bytes`, which
 * gives the HBM rate this GPU sustains for such a stream and a known-size reference for
 * scaling profiler byte counters.
 */
DDL_API ddl_status ddl_copy_probe(void* dst, const void* src, size_t bytes, void* hip_stream);

/*
 * Launch-shape knobs, for measurement; process-wide, read by every later call.  Names:
 *   "tiles_per_block"       consecutive 1024-element tiles one workgroup walks, 1..1024; -1
 *                           (default): one, two for 4-bit codes of more than eight learners
 *   "max_blocks_per_cu"     0: no cap; k in 3..64: at most k workgroups resident per compute
 *                           unit; -1 (default): chosen by learner type and count, 3 to 6
 *   "tile_rotate"           0: workgroup b takes run-of-tiles b; k in 2..4096: the index is
 *                           rotated within groups of k by the group's number, which spreads
 *                           every XCD's accesses over all memory channels (64)
 *   "max_tiles_per_launch"  a sync of more tiles than this goes out as several equal kernel
 *                           launches back to back, which keeps the eight XCDs aligned; 0: never
 *                           split; -1 (default): from "part_megabytes" and the bytes per tile
 *   "part_megabytes"        algorithmic traffic one such launch should carry, in 10^6 bytes,
 *                           1..1000000 (2500)
 *   "rda_blocks_per_cu"     residency cap of the RDA one-kernel shapes (0: none)
 *   "grids_enqueued"        read-only statistic: kernel launches this process has enqueued
 * Unknown name or bad value: INVALID_ARG.  ddl_get_option writes the current value.
 */
DDL_API ddl_status ddl_set_option(const char* name, long value);
DDL_API ddl_status ddl_get_option(const char* name, long* value_out);

#ifdef __cplusplus
}
#endif
#endif /* DDLSYNC_H */
