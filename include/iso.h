/*
 * iso.h -- C ABI of libiso: isomorphic sparse all-to-all and allgather on a
 * d-dimensional torus whose p processes are all virtual ranks resident in one
 * GPU's memory (gfx950).
 *
 * The interface follows the paper's persistent interface (Section 2: the
 * neighbourhood set-up call, the *_init calls, Iso_start, Iso_request_free;
 * Section 7: the proposed Iso_wait), with the MPI objects replaced by plain
 * arguments: torus dimension sizes, the flattened list of relative
 * coordinates, the block size in bytes, device pointers and a HIP stream.
 *
 * Conventions
 *   - Every function returns an int status: ISO_SUCCESS (0) or an ISO_ERR_*
 *     code.  No exception or abort crosses this boundary.  On error the output
 *     handle (if any) is left NULL.
 *   - Ranks are row-major over (p_0..p_{d-1}), last dimension fastest.
 *   - "host" / "device" below says where a pointer must live.  The caller owns
 *     every buffer it passes; the library owns only its handles and, per
 *     request, one small device table of block index maps (allocated in the
 *     init call, freed in iso_request_free).
 *   - A handle may be used from one host thread at a time.
 */
#ifndef ISO_H
#define ISO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ISO_MAX_DIMS 16          /* largest torus dimensionality accepted */

enum iso_status {
    ISO_SUCCESS       = 0,
    ISO_ERR_ARG       = 1,       /* null / out-of-range / inconsistent argument            */
    ISO_ERR_OVERLAP   = 2,       /* send, receive and workspace ranges are not disjoint     */
    ISO_ERR_WORKSPACE = 3,       /* workspace smaller than iso_workspace_bytes() reports    */
    ISO_ERR_HIP       = 4,       /* a HIP runtime call failed (see iso_last_hip_error)      */
    ISO_ERR_NOMEM     = 5,       /* host allocation failed                                  */
    ISO_ERR_TOO_LARGE = 6,       /* a size exceeds what the kernels index (see iso_*_init)  */
    ISO_ERR_POINTER   = 7,       /* a buffer is not device memory or its allocation is too
                                    small for the range the collective touches             */
    ISO_ERR_SCRATCH   = 8        /* iso_neighbor_alltoall_noalloc: the collective needs more
                                    than the library's static scratch memory holds         */
};

enum iso_op {
    ISO_OP_ALLTOALL  = 0,        /* individual block per neighbour (Section 2)  */
    ISO_OP_ALLGATHER = 1         /* same block to every neighbour (Section 2)   */
};

enum iso_algorithm {
    /* Message-combining, torus-direct schedule (Section 5): one round per
     * dimension j and distinct non-zero coordinate value v; one kernel launch
     * per round.  All-to-all uses the alternating receive/intermediate buffer
     * rule of Algorithm 1; allgather routes along the prefix trie of
     * Section 3.2. */
    ISO_ALG_COMBINED       = 0,
    /* Same schedule, all rounds of one dimension issued as a single launch
     * (they touch disjoint blocks; the k-ported remark of Section 3). */
    ISO_ALG_COMBINED_BYDIM = 1,
    /* Straightforward algorithm (first listing of Section 3): one exchange,
     * here one launch, per neighbour; s launches. */
    ISO_ALG_SX_ROUNDS      = 2,
    /* The same s exchanges issued as a single launch. */
    ISO_ALG_SX_FUSED       = 3,
    /* One-ported torus schedule (Sections 3.1-3.3, Algorithm 1 as printed): every
     * round moves blocks one hop along one dimension; per dimension max c_j
     * positive steps, then max -c_j negative steps, counted on the coordinates
     * as given (not reduced modulo p_j).  D = sum_j (max+ + max-) launches,
     * V = sum_i ||C^i||_1 block-moves per rank (all-to-all), W (allgather).
     * ISO_ERR_TOO_LARGE if D would exceed 65536. */
    ISO_ALG_ONEHOP         = 4,
    /* The message-combining schedule of ISO_ALG_COMBINED for small blocks in the
     * paper's [p][s][m] layout, where a round that writes a few blocks of every
     * rank's row costs far more memory traffic than the blocks hold.  The moves are
     * those of ISO_ALG_COMBINED (same sources, distances and dimensions, same
     * sum_i nnz(C^i) count for the all-to-all), the rounds of a dimension issued as
     * one launch as in ISO_ALG_COMBINED_BYDIM, but the receive buffer is written
     * by the last launch only: the last hop of every block is taken out of its round
     * and all of them run as one launch (ISO_ROUND_DELIVER) that gathers, through
     * LDS, every rank's s blocks and writes whole receive rows.  A move into the
     * receive buffer that cannot wait (its block is read again, or its source is
     * overwritten later: allgather trie nodes) goes to an extra workspace slot and is
     * copied from there by the last launch; the workspace grows by one plane of
     * p*m bytes per such block.  Rounds left empty disappear.  The row-writing
     * launch takes equal blocks that are multiples of 16 bytes in dense rank-major
     * rows with s <= 128 and s*m <= 32 KiB; any other request runs the same plan on
     * the general kernels, the last launch as one launch per dimension (so the
     * request's launches can exceed the plan's rounds).  Not available on a mesh
     * (ISO_ERR_ARG). */
    ISO_ALG_COMBINED_STAGED = 5
};

enum iso_buffer {                /* where a block sits during a schedule */
    ISO_BUF_SEND = 0,
    ISO_BUF_RECV = 1,
    ISO_BUF_WORK = 2             /* intermediate buffer (all-to-all, Algorithm 1) or
                                    temporary trie nodes (allgather) in the workspace */
};

enum iso_round_kind {
    ISO_ROUND_SHIFT  = 0,        /* every entry moves along one dimension (per-entry distance) */
    ISO_ROUND_SELF   = 1,        /* zero offset: same-rank copy send -> recv                   */
    ISO_ROUND_VECTOR = 2,        /* every entry moves by its full offset vector (s-exchange)   */
    ISO_ROUND_DELIVER = 3        /* last launch of ISO_ALG_COMBINED_STAGED: entry i writes receive
                                    block i; every entry moves along its own dimension
                                    (iso_plan_entry_t.dim, -1: same-rank copy)                 */
};

enum iso_layout {                /* how the p*s blocks of a regular collective lie in a buffer  */
    /* the paper's layout (Section 2): every process holds its s blocks back to
     * back in neighbour order, processes back to back: [p][s][m]                */
    ISO_LAYOUT_RANK_MAJOR = 0,
    /* one plane per neighbour: block i of all processes back to back, planes in
     * neighbour order: [s][p][m].  Every block-move of a round then reads and
     * writes a dense stream whatever m is (the layout the workspace always has). */
    ISO_LAYOUT_SLOT_MAJOR = 1
};

typedef struct iso_comm_s    *iso_comm_t;     /* torus + neighbourhood                    */
typedef struct iso_plan_s    *iso_plan_t;     /* schedule for (comm, op, algorithm)       */
typedef struct iso_request_s *iso_request_t;  /* schedule bound to buffers and block size */

typedef struct {
    int32_t d;                   /* dimensions                                             */
    int32_t s;                   /* neighbours                                             */
    int64_t p;                   /* processes = prod p_j                                   */
    int32_t rounds;              /* torus-direct rounds: sum_j #distinct non-zero residues */
    int32_t self_slots;          /* neighbours whose offset is 0 modulo the torus          */
    int64_t alltoall_moves;      /* sum_i nnz(C^i): blocks moved per rank, all-to-all      */
    int64_t allgather_moves;     /* blocks moved per rank, allgather (trie, chosen order)  */
} iso_comm_info_t;

typedef struct {
    int32_t op, algorithm;
    int32_t launches;            /* kernel launches per iso_start (= rounds of the plan)   */
    int32_t work_slots;          /* blocks per rank held in the workspace                  */
    int64_t entries;             /* block-moves per rank per collective (incl. self)       */
    int32_t dim_order[ISO_MAX_DIMS]; /* allgather: order in which dimensions are routed    */
} iso_plan_info_t;

typedef struct {
    int32_t kind;                /* enum iso_round_kind                                    */
    int32_t dim;                 /* ISO_ROUND_SHIFT: dimension j; otherwise -1             */
    int32_t n_entries;           /* k: blocks moved per rank in this launch                */
    int32_t reserved;
} iso_round_info_t;

typedef struct {
    int32_t src_buf, src_slot;   /* enum iso_buffer, block index inside that buffer's row  */
    int32_t dst_buf, dst_slot;
    int32_t shift;               /* SHIFT rounds: the block comes from the rank `shift` steps
                                    back in `dim`.  Periodic dimension: the residue v in
                                    [0, p_j).  Non-periodic dimension of a mesh: the signed
                                    coordinate as given (negative = the source lies forward,
                                    magnitudes of p_j and more are legal and find no source
                                    anywhere).  Other rounds: 0                            */
    int32_t neighbor;            /* index i of the offset whose route this move belongs to
                                    (allgather temporaries: -1); VECTOR rounds: source is
                                    R (-) C^neighbor                                        */
    int32_t ref;                 /* a neighbour whose route passes through this move (always
                                    valid; equals `neighbor` when that is >= 0).  On a mesh
                                    the move happens at rank R only if R minus C^ref, taken
                                    over the dimensions routed so far, is inside the mesh    */
    int32_t dim;                 /* the dimension the move runs along: the round's for SHIFT
                                    rounds, the entry's own in a DELIVER round; -1 where the
                                    entry is a same-rank copy or moves by a full vector     */
} iso_plan_entry_t;

typedef struct {
    int32_t op, algorithm;
    int32_t launches;
    int32_t vector_bytes;        /* width of the loads/stores: the largest power of two that is
                                  * at most 16 and at most the smallest non-empty block; buffer
                                  * addresses need no alignment                               */
    int64_t p, s;
    uint64_t block_bytes;        /* m                                                       */
    int64_t entries;             /* block-moves per rank                                    */
    uint64_t bytes_read;         /* algorithmic bytes read per iso_start = entries*p*m      */
    uint64_t bytes_written;      /* algorithmic bytes written per iso_start                 */
    uint64_t delivered_bytes;    /* p*s*m                                                   */
    uint64_t workspace_bytes;    /* workspace the request uses                              */
} iso_request_info_t;

/* ---- neighbourhood set-up (Section 2, set-up listing) ----------------------
 * dims:       host, d ints, every p_j >= 1, 1 <= d <= ISO_MAX_DIMS, prod < 2^31.
 * rel_coords: host, s*d ints, neighbour-major: C^0_0..C^0_{d-1}, C^1_0, ...
 *             Arbitrary signed values, repeats and the zero vector are legal;
 *             coordinates are reduced modulo p_j.  s >= 0.
 * The arrays are copied; the order of the s vectors fixes the block order in
 * the send and receive buffers.  Purely local host computation, O(s d). */
int iso_neighborhood_create(int d, const int32_t *dims, int s,
                            const int32_t *rel_coords, iso_comm_t *comm);
/* Same, on a mesh (Section 7: non-periodic dimensions, as in an MPI Cartesian
 * topology).  periodic: host, d flags (non-zero = the dimension wraps); NULL =
 * all periodic = iso_neighborhood_create.  In a non-periodic dimension
 * coordinates are taken as given (not reduced) and nothing wraps: a rank whose
 * source R - C^i lies outside the mesh receives nothing for neighbour i and its
 * i-th receive block keeps its content.  Intermediate hops of the all-to-all
 * then alternate between two workspace slots instead of using the receive
 * buffer, so that blocks in transit never overwrite a block that stays
 * untouched.  ISO_ALG_ONEHOP is not available on a mesh (ISO_ERR_ARG). */
int iso_neighborhood_create_mesh(int d, const int32_t *dims, const int32_t *periodic, int s,
                                 const int32_t *rel_coords, iso_comm_t *comm);
int iso_neighborhood_info(iso_comm_t comm, iso_comm_info_t *info);
/* Frees the handle and sets *comm = NULL.  Plans and requests made from it
 * keep their own copy of what they need and stay valid. */
int iso_neighborhood_free(iso_comm_t *comm);

/* ---- schedules, host only (Algorithm 1; Sections 3.2 and 5) ----------------
 * A plan lists, per launch, the block-moves every rank performs.  No device is
 * touched: these calls work without a GPU and exist so that a schedule can be
 * inspected and checked. */
int iso_plan_create(iso_comm_t comm, int op, int algorithm, iso_plan_t *plan);
int iso_plan_info(iso_plan_t plan, iso_plan_info_t *info);
int iso_plan_round(iso_plan_t plan, int round, iso_round_info_t *info);
/* Copies min(capacity, n_entries) entries of `round` to host array `out`. */
int iso_plan_entries(iso_plan_t plan, int round, iso_plan_entry_t *out, int capacity);
int iso_plan_free(iso_plan_t *plan);

/* Bytes of device workspace an init call with these arguments needs (may be 0).
 * All-to-all: the intermediate buffer of Algorithm 1, restricted to the blocks
 * that make two or more hops.  Allgather: trie nodes that are not themselves
 * neighbours.  The s-exchange algorithms need none. */
int iso_workspace_bytes(iso_comm_t comm, int op, int algorithm, size_t m, size_t *bytes);
/* The same for the message-combining schedule (ISO_ALG_COMBINED) of one operation:
 * iso_workspace_bytes(comm, ISO_OP_ALLTOALL / ISO_OP_ALLGATHER, ISO_ALG_COMBINED, m, bytes). */
int iso_alltoall_workspace_bytes(iso_comm_t comm, size_t m, size_t *bytes);
int iso_allgather_workspace_bytes(iso_comm_t comm, size_t m, size_t *bytes);

/* ---- persistent collectives (Section 2, init/start listing) ----------------
 * sendbuf:   device, read-only.  All-to-all: p*s blocks, [p][s][m], block (R,i)
 *            is what rank R sends to rank R (+) C^i.  Allgather: [p][m].
 * recvbuf:   device, [p][s][m]; after completion block (R,i) holds what rank
 *            R (-) C^i sent (all-to-all: its i-th block; allgather: its block).
 * m:         block size in bytes, any value >= 0 (m == 0 or s == 0: no-op).
 *            Loads and stores are 16 bytes wide for m >= 16 (below: the largest
 *            power of two that is at most m); the buffers need no alignment.
 *            Blocks whose ends fall on 32-byte boundaries are written fastest.
 * workspace: device, at least iso_workspace_bytes() bytes (NULL allowed when
 *            that is 0).  Contents are scratch while a collective runs.
 * The three ranges must not overlap (ISO_ERR_OVERLAP); in-place operation is
 * not supported.  Each must lie inside one device allocation (ISO_ERR_POINTER).
 * ISO_ERR_TOO_LARGE if p*m >= 2^36 (one block plane would exceed what a launch
 * indexes) or if consecutive ranks' blocks are 2^32 bytes or more apart (s*m here,
 * an extent in the irregular calls).  The buffers are bound to the request; iso_start may be called any
 * number of times.  Needs a GPU (uploads the index maps: one hipMalloc + one
 * synchronous hipMemcpy). */
int iso_neighbor_alltoall_init(const void *sendbuf, void *recvbuf, size_t m,
                               void *workspace, size_t workspace_bytes,
                               iso_comm_t comm, int algorithm, iso_request_t *req);
int iso_neighbor_allgather_init(const void *sendbuf, void *recvbuf, size_t m,
                                void *workspace, size_t workspace_bytes,
                                iso_comm_t comm, int algorithm, iso_request_t *req);

/* The straightforward algorithm (first listing of Section 3: one exchange per
 * neighbour) bound as a persistent request: the comparison baseline.
 * mode: ISO_SX_LAUNCHES = one launch per neighbour, s launches (the listing taken
 * literally; = ISO_ALG_SX_ROUNDS), ISO_SX_FUSED = all s exchanges in one launch
 * (= ISO_ALG_SX_FUSED).  No workspace is needed.  Buffers, layout ([p][s][m]),
 * results and errors as for iso_neighbor_alltoall_init / _allgather_init. */
enum iso_sx_mode { ISO_SX_LAUNCHES = 0, ISO_SX_FUSED = 1 };
int iso_neighbor_alltoall_sx_init(const void *sendbuf, void *recvbuf, size_t m, int mode,
                                  iso_comm_t comm, iso_request_t *req);
int iso_neighbor_allgather_sx_init(const void *sendbuf, void *recvbuf, size_t m, int mode,
                                   iso_comm_t comm, iso_request_t *req);

/* The same two collectives with the layout of the caller's buffers chosen by
 * `layout` (enum iso_layout).  ISO_LAYOUT_RANK_MAJOR is exactly the calls above.
 * ISO_LAYOUT_SLOT_MAJOR: sendbuf (all-to-all) and recvbuf are [s][p][m]: block
 * (R,i) sits at offset (i*p + R)*m; the allgather sendbuf stays [p][m].  Results
 * are the same blocks at their new places: recv(R,i) = send(R (-) C^i, i).  All
 * other rules (alignment, overlap, workspace size, errors) are unchanged. */
int iso_neighbor_alltoall_init_layout(const void *sendbuf, void *recvbuf, size_t m, int layout,
                                      void *workspace, size_t workspace_bytes,
                                      iso_comm_t comm, int algorithm, iso_request_t *req);
int iso_neighbor_allgather_init_layout(const void *sendbuf, void *recvbuf, size_t m, int layout,
                                       void *workspace, size_t workspace_bytes,
                                       iso_comm_t comm, int algorithm, iso_request_t *req);

/* ---- irregular variants (Section 2, second interface listing) ---------------
 * Per-neighbour block sizes and displacements, in bytes, the same on every
 * rank; the paper's v and w variants differ only in MPI datatypes and collapse
 * into this one byte-based form.  The same schedules are used (Section 4).
 *   send_sizes/recv_sizes: host, s values; must be equal pairwise (ISO_ERR_ARG).
 *   send_displs/recv_displs: host, s values: offset of block i inside a rank's row.
 *   send_extent/recv_extent: bytes between the rows of consecutive ranks; every
 *     block must lie inside its row (ISO_ERR_ARG); receive blocks must not
 *     overlap each other (ISO_ERR_OVERLAP); send blocks may.
 *   sendbuf: device, rank R's row starts at sendbuf + R*send_extent (read-only);
 *   recvbuf: device, likewise; bytes of a row outside the s blocks are not touched.
 * Blocks of size 0 are legal and move nothing.  Each block is moved in units of
 * its own width: 16 bytes for blocks of 16 bytes and more, below that the largest
 * power of two that is at most the block size (the last unit of a block overlaps
 * its predecessor when the width does not divide the size), so a 1-byte block
 * next to a 16 KiB block does not narrow the latter.  Addresses, displacements
 * and extents need no alignment; rows whose blocks start on 128-byte boundaries
 * are written fastest.
 * Workspace: iso_workspace_bytes_v() (sizes: host, s values; for ISO_OP_ALLGATHER
 * they must all be equal, as in the init call, else ISO_ERR_ARG).  Other rules as
 * for the regular calls. */
int iso_workspace_bytes_v(iso_comm_t comm, int op, int algorithm, const size_t *sizes, size_t *bytes);
int iso_neighbor_alltoallv_init(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs,
                                size_t send_extent, void *recvbuf, const size_t *recv_sizes,
                                const size_t *recv_displs, size_t recv_extent, void *workspace,
                                size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                iso_request_t *req);
/* Allgather: every rank contributes one block of send_size bytes (its row starts at
 * sendbuf + R*send_extent); recv_sizes must all equal send_size (ISO_ERR_ARG). */
int iso_neighbor_allgatherv_init(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                                 const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                                 void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                 iso_request_t *req);

/* The irregular calls with the layout of the caller's buffers chosen by `layout`.
 * ISO_LAYOUT_RANK_MAJOR: exactly the calls above.  ISO_LAYOUT_SLOT_MAJOR: one
 * plane per neighbour; block i of rank R sits at displs[i] + R * sizes[i], plane i
 * covers [displs[i], displs[i] + p * sizes[i]); the extents are ignored except
 * send_extent of the allgather, whose send buffer stays one row per rank.  Receive
 * planes must not overlap (ISO_ERR_OVERLAP). */
int iso_neighbor_alltoallv_init_layout(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs,
                                       size_t send_extent, void *recvbuf, const size_t *recv_sizes,
                                       const size_t *recv_displs, size_t recv_extent, int layout,
                                       void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                       iso_request_t *req);
int iso_neighbor_allgatherv_init_layout(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                                        const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                                        int layout, void *workspace, size_t workspace_bytes, iso_comm_t comm,
                                        int algorithm, iso_request_t *req);

/* The paper's w variants (per-neighbour datatypes, displacements in bytes): with
 * every size and displacement already in bytes they are the v calls under their
 * second name; same arguments, same behaviour. */
int iso_neighbor_alltoallw_init(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs,
                                size_t send_extent, void *recvbuf, const size_t *recv_sizes,
                                const size_t *recv_displs, size_t recv_extent, void *workspace,
                                size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                iso_request_t *req);
int iso_neighbor_allgatherw_init(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                                 const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                                 void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                 iso_request_t *req);

/* Enqueues the launches of one collective on `hip_stream` (a hipStream_t; NULL
 * = the default stream) and returns without waiting.  Rounds are ordered by the
 * stream.  Calls on one request must not overlap in time on the device. */
int iso_start(iso_request_t req, void *hip_stream);
/* Enqueues only launches [first, first+count) of the request's launch list, in
 * order (0 <= first, first+count <= launches of iso_request_info).  For timing
 * individual rounds; running all ranges in order equals one iso_start. */
int iso_start_range(iso_request_t req, int first, int count, void *hip_stream);
/* Replays the request's launches as a HIP graph: the persistent request of
 * Section 2 taken one step further, for collectives whose cost is dominated by
 * the per-round start-up.  enable (enum iso_graph_form):
 *   ISO_GRAPH_OFF      back to individual launches;
 *   ISO_GRAPH_CHAIN    one kernel node per launch, each after the one before;
 *   ISO_GRAPH_BRANCHES one kernel node per launch with an edge only where a later
 *                      launch reads or overwrites blocks an earlier one wrote, or
 *                      overwrites blocks it read: the rounds of one dimension,
 *                      which move disjoint blocks, become parallel branches.
 * The graph is built on the first call that asks for a form and replayed by every
 * later iso_start with one hipGraphLaunch; asking for the other form waits for
 * the request's last start and rebuilds.  iso_start_range is unaffected.  The
 * result is the same in every form.  (On the ROCm 7.2 runtime neither form is
 * faster than individual launches: a graph launch costs more than the launches
 * it replaces, and every join of branches adds 8 to 20 microseconds.) */
enum iso_graph_form { ISO_GRAPH_OFF = 0, ISO_GRAPH_CHAIN = 1, ISO_GRAPH_BRANCHES = 2 };
int iso_request_set_graph(iso_request_t req, int enable);
/* Blocks the host until the most recent iso_start / iso_start_range of this
 * request completed (Section 7's proposed completion call).  Only the stream of
 * that most recent call is waited for: a caller that starts ranges of one request
 * on several streams synchronises the earlier streams itself. */
int iso_wait(iso_request_t req);
int iso_request_info(iso_request_t req, iso_request_info_t *info);
/* Returns the plan the request executes (owned by the request; do not free). */
int iso_request_plan(iso_request_t req, iso_plan_t *plan);
/* Waits for the request's most recent start (as iso_wait does), then frees the
 * handle, its graph and its device table, and sets *req = NULL. */
int iso_request_free(iso_request_t *req);

/* ---- for callers that cannot allocate device memory -------------------------
 * Code under HIP graph capture, tight serving loops and harnesses that forbid
 * hipMalloc cannot use the init calls (they allocate the request's device
 * table) and may have no workspace to pass.  This call is
 * iso_neighbor_alltoall_init + iso_start in one, with no request left behind:
 * it enqueues one all-to-all (same arguments, layout [p][s][m], same result,
 * same algorithms) on `hip_stream` and returns without waiting.  The table of
 * block index maps and the intermediate buffer live in a static device array
 * of ISO_NOALLOC_SCRATCH_BYTES that each GPU holds from the moment the
 * library's code is loaded on it until the process ends; the table is written
 * by small kernels that carry it in their arguments, ordered on the stream
 * before the rounds.  No hipMalloc, hipFree, host-to-device copy or other
 * allocating routine is called.
 * Limits: the table (48 bytes per block-move per rank, plus 4*s*d) must fit
 * ISO_NOALLOC_TABLE_BYTES and iso_workspace_bytes() the rest of the array,
 * else ISO_ERR_SCRATCH and nothing is enqueued.
 * All calls on one GPU share that GPU's array, which keeps the previous call's
 * contents (nothing in it needs to start at zero: every block of the
 * intermediate buffer is written before it is read, and the table is rewritten
 * by every call).  Calls follow each other safely on one stream; calls that
 * overlap in time on one GPU (different streams, different threads) race. */
#define ISO_NOALLOC_SCRATCH_BYTES (32u << 20)
#define ISO_NOALLOC_TABLE_BYTES   (256u << 10)
int iso_neighbor_alltoall_noalloc(const void *sendbuf, void *recvbuf, size_t m, iso_comm_t comm,
                                  int algorithm, void *hip_stream);

/* ---- diagnostics ----------------------------------------------------------- */
const char *iso_error_string(int status);
/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int iso_last_hip_error(void);
/* Plain device-to-device copy of `bytes` bytes with the library's streaming
 * kernel (16-byte accesses when alignment allows): the bandwidth ceiling that
 * the round kernels are measured against.  src/dst: device, non-overlapping. */
int iso_copy_reference(const void *src, void *dst, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ISO_H */
